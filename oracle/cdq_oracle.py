"""Python face of the CPU oracle.  TEST INFRASTRUCTURE ONLY.

Only tests, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg may
import this.  It never touches the HIP library or the GPU.

Steps whose plain definition is a library primitive use numpy in fp64 (the
Hessian X^T X); the order-sensitive and fp32-canonical steps are the scalar C
loops of ``cdq_oracle.c``.  See that file's header for conventions, readings
and the list of pins.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cdq_oracle.c")
_SO = os.path.join(_HERE, "libcdq_oracle.so")
_lib = None


def _host_has_fma() -> bool:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("flags"):
                    return " fma " in line + " "
    except OSError:
        pass
    return False


def build(force: bool = True) -> str:
    """Compile cdq_oracle.c with gcc.  -ffp-contract=off: every fused multiply-add
    in the oracle is an explicit fmaf(); -mfma only lets gcc inline those calls."""
    if not force and os.path.exists(_SO) and os.path.getmtime(_SO) >= os.path.getmtime(_SRC):
        return _SO
    cmd = ["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
           "-shared", "-fPIC", _SRC, "-o", _SO, "-lm"]
    if _host_has_fma():
        cmd.insert(1, "-mfma")
    subprocess.run(cmd, check=True)
    return _SO


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        if not _host_has_fma():
            build(force=True)       # a library built elsewhere with -mfma would not run here
        _lib = ctypes.CDLL(_SO)
    return _lib


def n_threads() -> int:
    """Threads the OpenMP loops over columns will use."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        try:
            return max(1, int(env.split(",")[0]))
        except ValueError:
            pass
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


_I64 = ctypes.c_int64


# --------------------------------------------------------------------------- Hessian

def hessian(X, lambda_rel: float = 0.0) -> np.ndarray:
    """H = X^T X in fp64 (Section 3, Notation; Algorithm 1 'Compute Hessian'), plus the
    damping lambda*I of Section 4 ('Baselines'/'CDQuant') parameterised as
    lambda = lambda_rel * mean(diag H) because the paper does not give its value."""
    X64 = np.asarray(X, dtype=np.float64)
    H = X64.T @ X64
    if lambda_rel:
        H[np.diag_indices_from(H)] += lambda_rel * float(np.mean(np.diag(H)))
    return H


# --------------------------------------------------------------------------- grid / RTN (Eq. 2)

def init_grid(Wt, bits: int, group: int, gamma=1.0):
    """Eq. (2) in fp32, per (column, group): b = min w, a = gamma (max w - min w)/(2^c - 1),
    q = clamp(round_half_even((w - b)/a), 0, 2^c - 1).  gamma = 1 is MinMax
    round-to-nearest.  gamma may be a scalar or an array [d_out][n_grp].
    A constant group (a == 0) gets a = 1, q = 0, which reproduces w exactly."""
    Wt = np.ascontiguousarray(Wt, dtype=np.float32)
    d_out, d_in = Wt.shape
    assert d_in % group == 0
    n_grp = d_in // group
    L1 = np.float32((1 << bits) - 1)
    Wg = Wt.reshape(d_out, n_grp, group)
    lo = Wg.min(axis=2)
    hi = Wg.max(axis=2)
    gam = np.broadcast_to(np.asarray(gamma, dtype=np.float32), (d_out, n_grp))
    a = ((gam * (hi - lo)).astype(np.float32) / L1).astype(np.float32)
    a = np.where((a > 0) & np.isfinite(a), a, np.float32(1.0)).astype(np.float32)
    b = lo.astype(np.float32)
    t = ((Wg - b[:, :, None]).astype(np.float32) / a[:, :, None]).astype(np.float32)
    q = np.clip(np.rint(t), np.float32(0), L1)
    return a, b, q.reshape(d_out, d_in).astype(np.uint8)


# --------------------------------------------------------------------------- residual, gradient, loss

def residual(Wt, Q, scale, zero, group: int, precision: str = "f32") -> np.ndarray:
    lib = _load()
    d_out, d_in = Q.shape
    Q = np.ascontiguousarray(Q, np.uint8)
    dt = np.float32 if precision == "f32" else np.float64
    Wt, scale, zero = (np.ascontiguousarray(x, dt) for x in (Wt, scale, zero))
    E = np.empty((d_out, d_in), dt)
    fn = lib.cdqo_residual_f32 if precision == "f32" else lib.cdqo_residual_f64
    fn(_p(Wt), _p(Q), _p(scale), _p(zero), _I64(d_out), _I64(d_in), _I64(group), _p(E))
    return E


def gradient(H, E, precision: str = "f32") -> np.ndarray:
    """g_j = H e_j for every column.  f32: fp32 H and e, fp64 running sum, one rounding."""
    lib = _load()
    d_out, d_in = E.shape
    dt = np.float32 if precision == "f32" else np.float64
    H = np.ascontiguousarray(H, dt)
    E = np.ascontiguousarray(E, dt)
    G = np.empty((d_out, d_in), dt)
    fn = lib.cdqo_gradient_f32 if precision == "f32" else lib.cdqo_gradient_f64
    fn(_p(H), _p(E), _I64(d_out), _I64(d_in), _p(G))
    return G


def loss(H, Wt, Q, scale, zero, group: int) -> np.ndarray:
    """Per-column loss e^T H e of Eq. (1) in fp64 (inputs are promoted exactly)."""
    lib = _load()
    E = residual(Wt, Q, scale, zero, group, "f64")
    H = np.ascontiguousarray(H, np.float64)
    d_out, d_in = E.shape
    out = np.empty(d_out, np.float64)
    lib.cdqo_loss_f64(_p(H), _p(E), _I64(d_out), _I64(d_in), _p(out))
    return out


# --------------------------------------------------------------------------- greedy CD

def greedy_cd(H, Wt, scale, zero, Q0, bits: int, group: int, T: int,
              precision: str = "f32", trace_cap: int = 0):
    """Algorithm 1 (Algorithm 4 when group < d_in) for every column.  Returns a dict with
    Q (final codes), moves, converged, G (final g = H e as maintained by the updates) and,
    if trace_cap > 0, trace_i / trace_r / trace_s of the committed moves."""
    lib = _load()
    Q = np.ascontiguousarray(Q0, np.uint8).copy()
    d_out, d_in = Q.shape
    assert d_in % group == 0
    dt = np.float32 if precision == "f32" else np.float64
    H = np.ascontiguousarray(H, dt)
    assert H.shape == (d_in, d_in)
    scale = np.ascontiguousarray(scale, dt)
    E = residual(Wt, Q, scale, zero, group, precision)
    G = gradient(H, E, precision)
    moves = np.zeros(d_out, np.int32)
    conv = np.zeros(d_out, np.int32)
    cap = max(int(trace_cap), 0)
    ti = np.full((d_out, max(cap, 1)), -1, np.int32)
    tr = np.full((d_out, max(cap, 1)), -1, np.int32)
    ts = np.zeros((d_out, max(cap, 1)), dt)
    fn = lib.cdqo_greedy_cd_f32 if precision == "f32" else lib.cdqo_greedy_cd_f64
    fn(_p(H), _p(scale), _p(Q), _p(G), _I64(d_out), _I64(d_in), ctypes.c_int(bits), _I64(group), _I64(T),
       _p(moves), _p(conv), _p(ti), _p(tr), _p(ts), _I64(cap))
    out = {"Q": Q, "moves": moves, "converged": conv, "G": G}
    if cap:
        out.update(trace_i=ti, trace_r=tr, trace_s=ts)
    return out


def argmin_step(Hdiag, scale, Q, G, bits: int, group: int):
    """One arg-min step of Algorithm 1 on given (Q, G): per column (i*, r*, s*), i* = -1 if none < 0."""
    lib = _load()
    Q = np.ascontiguousarray(Q, np.uint8)
    d_out, d_in = Q.shape
    Hdiag, scale, G = (np.ascontiguousarray(x, np.float32) for x in (Hdiag, scale, G))
    oi = np.empty(d_out, np.int32)
    orr = np.empty(d_out, np.int32)
    os_ = np.empty(d_out, np.float32)
    lib.cdqo_argmin_f32(_p(Hdiag), _p(scale), _p(Q), _p(G), _I64(d_out), _I64(d_in), ctypes.c_int(bits),
                        _I64(group), _p(oi), _p(orr), _p(os_))
    return oi, orr, os_


def cyclic_cd(H, Wt, scale, zero, Q0, bits: int, group: int, T: int, trace_cap: int = 0):
    """Cyclic (fixed-order) coordinate descent in canonical fp32: visit t handles coordinate t mod d_in; T visits at
    most; stops once d_in consecutive visits made no move.  Returns Q, moves, iters, converged, G[, trace_*]."""
    lib = _load()
    Q = np.ascontiguousarray(Q0, np.uint8).copy()
    d_out, d_in = Q.shape
    assert d_in % group == 0
    H = np.ascontiguousarray(H, np.float32)
    scale = np.ascontiguousarray(scale, np.float32)
    E = residual(Wt, Q, scale, zero, group, "f32")
    G = gradient(H, E, "f32")
    moves, iters, conv = (np.zeros(d_out, np.int32) for _ in range(3))
    cap = max(int(trace_cap), 0)
    ti = np.full((d_out, max(cap, 1)), -1, np.int32)
    tr = np.full((d_out, max(cap, 1)), -1, np.int32)
    ts = np.zeros((d_out, max(cap, 1)), np.float32)
    lib.cdqo_cyclic_cd_f32(_p(H), _p(scale), _p(Q), _p(G), _I64(d_out), _I64(d_in), ctypes.c_int(bits), _I64(group), _I64(T),
                           _p(moves), _p(iters), _p(conv), _p(ti), _p(tr), _p(ts), _I64(cap))
    out = {"Q": Q, "moves": moves, "iters": iters, "converged": conv, "G": G}
    if cap:
        out.update(trace_i=ti, trace_r=tr, trace_s=ts)
    return out


def bcd(H, Wt, scale, zero, Q0, parts, bits: int, group: int, k: int = 2, trace_cap: int = 0):
    """Algorithm 2 (Algorithm 5 when group < d_in) in canonical fp32 for every column, block size k.
    parts [T][d_in] int32: row t is the random partition of iteration t, block b = parts[t, k*b : k*b+k].
    Returns Q, moves, G and, if trace_cap > 0, trace_t (iteration), trace_b (block), trace_r (levels,
    4 bits per member, member 0 lowest), trace_s."""
    lib = _load()
    Q = np.ascontiguousarray(Q0, np.uint8).copy()
    d_out, d_in = Q.shape
    parts = np.ascontiguousarray(parts, np.int32)
    T = parts.shape[0]
    assert parts.shape == (T, d_in) and d_in % k == 0 and d_in % group == 0 and 1 <= k <= 8
    assert (np.sort(parts, axis=1) == np.arange(d_in)).all(), "every row of parts must be a permutation"
    H = np.ascontiguousarray(H, np.float32)
    scale = np.ascontiguousarray(scale, np.float32)
    E = residual(Wt, Q, scale, zero, group, "f32")
    G = gradient(H, E, "f32")
    moves = np.zeros(d_out, np.int32)
    cap = max(int(trace_cap), 0)
    tt, tb, tr = (np.full((d_out, max(cap, 1)), -1, np.int32) for _ in range(3))
    ts = np.zeros((d_out, max(cap, 1)), np.float32)
    lib.cdqo_bcd_f32(_p(H), _p(scale), _p(Q), _p(G), _p(parts), _I64(d_out), _I64(d_in), ctypes.c_int(bits), _I64(group),
                     ctypes.c_int(k), _I64(T), _p(moves), _p(tt), _p(tb), _p(tr), _p(ts), _I64(cap))
    out = {"Q": Q, "moves": moves, "G": G}
    if cap:
        out.update(trace_t=tt, trace_b=tb, trace_r=tr, trace_s=ts)
    return out


# --------------------------------------------------------------------------- OWC (Eq. 2 + grid search)

def owc_gammas(n_gamma: int = 50) -> np.ndarray:
    """Clipping-strength grid: the paper says only 'grid size 50' on [0,1] (Section 4,
    'Training'); this build reads it as k/n for k = 1..n, so 1 (MinMax) is in and 0 is out."""
    return (np.arange(1, n_gamma + 1, dtype=np.float32) / np.float32(n_gamma)).astype(np.float32)


def init_owc(H, Wt, bits: int, group: int, n_gamma: int = 50):
    """Optimal Weight Clipping for per-channel grids (Section 3.1, 'Initializing a, b, q'):
    for every gamma on the grid quantize with Eq. (2) and keep, per column, the gamma with
    the smallest loss of Eq. (1).  Equal losses keep the larger gamma.  Returns
    (scale, zero, Q, gamma, loss_per_gamma[n_gamma][d_out])."""
    Wt = np.ascontiguousarray(Wt, np.float32)
    d_out, d_in = Wt.shape
    assert group == d_in, "OWC as defined by Eq. (2) has one clipping strength per column"
    gammas = owc_gammas(n_gamma)
    best_loss = np.full(d_out, np.inf)
    best = None
    all_loss = np.empty((n_gamma, d_out))
    for k, gam in enumerate(gammas):
        a, b, q = init_grid(Wt, bits, group, gam)
        l = loss(H, Wt, q, a, b, group)
        all_loss[k] = l
        take = l <= best_loss
        if best is None:
            best = [a.copy(), b.copy(), q.copy(), np.full(d_out, gam, np.float32)]
        else:
            best[0][take] = a[take]
            best[1][take] = b[take]
            best[2][take] = q[take]
            best[3][take] = gam
        best_loss = np.where(take, l, best_loss)
    return best[0], best[1], best[2], best[3], all_loss


# --------------------------------------------------------------------------- OWC-CD (Algorithm 3)

def owc_cd(H, Wt, bits: int, group: int, n_gamma: int = 50, T: int | None = None, trace_cap: int = 0):
    """Greedy coordinate descent over per-group clipping strengths (Algorithm 3), every group
    starting at gamma = 1.  T defaults to d_in/group as in Section 4.  Returns a dict with scale,
    zero [d_out][n_grp], Q, gamma_idx (grid index k, gamma = k/n_gamma), moves, converged and the
    optional trace (trace_i = group, trace_r = grid index, trace_s = fp64 score)."""
    lib = _load()
    Wt = np.ascontiguousarray(Wt, np.float32)
    H = np.ascontiguousarray(H, np.float32)
    d_out, d_in = Wt.shape
    assert d_in % group == 0
    n_grp = d_in // group
    if T is None:
        T = n_grp
    scale = np.empty((d_out, n_grp), np.float32)
    zero = np.empty((d_out, n_grp), np.float32)
    Q = np.empty((d_out, d_in), np.uint8)
    gidx = np.zeros((d_out, n_grp), np.int32)
    moves = np.zeros(d_out, np.int32)
    conv = np.zeros(d_out, np.int32)
    cap = max(int(trace_cap), 0)
    ti = np.full((d_out, max(cap, 1)), -1, np.int32)
    tr = np.full((d_out, max(cap, 1)), -1, np.int32)
    ts = np.zeros((d_out, max(cap, 1)), np.float64)
    lib.cdqo_owc_cd(_p(H), _p(Wt), _I64(d_out), _I64(d_in), ctypes.c_int(bits), _I64(group), ctypes.c_int(n_gamma),
                    _I64(T), _p(scale), _p(zero), _p(Q), _p(gidx), _p(moves), _p(conv), _p(ti), _p(tr), _p(ts), _I64(cap))
    out = {"scale": scale, "zero": zero, "Q": Q, "gamma_idx": gidx, "moves": moves, "converged": conv}
    if cap:
        out.update(trace_i=ti, trace_r=tr, trace_s=ts)
    return out
