"""Thin binding over libcdq.so (see include/cdq.h).  Argument marshalling only: every step of
the path runs in the HIP kernels.  torch is used for device memory and streams, nothing else.

There is no fallback: if the library is missing or a call fails, this raises."""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libcdq.so")

CDQ_F32, CDQ_BF16 = 0, 1
OP_HESSIAN, OP_GREEDY_CD, OP_LOSS, OP_INIT_OWC, OP_INIT_OWC_CD, OP_BCD, OP_CYCLIC_CD = 0, 1, 2, 3, 4, 5, 6
MAX_D_IN = 36864

_lib = None


class CdqError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: cdq error {code}: {lib().cdq_strerror(code).decode()}")


class ColStats(ctypes.Structure):
    _fields_ = [("moves", ctypes.c_int32), ("iters", ctypes.c_int32), ("converged", ctypes.c_int32),
                ("last_score", ctypes.c_float)]


class CdOptions(ctypes.Structure):
    _fields_ = [("waves_per_column", ctypes.c_int32), ("elems_per_lane", ctypes.c_int32),
                ("exact_scorer_only", ctypes.c_int32), ("teams_per_cu", ctypes.c_int32),
                ("trace", ctypes.c_void_p), ("trace_cap", ctypes.c_int64), ("G_out", ctypes.c_void_p),
                ("ev_loop_begin", ctypes.c_void_p), ("ev_loop_end", ctypes.c_void_p), ("G0", ctypes.c_void_p)]


def lib() -> ctypes.CDLL:
    """Load libcdq.so; build it in-tree first if it is not there (needs hipcc)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            from . import build as _build
            _build.build()
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, i32, f32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
        L.cdq_strerror.restype = ctypes.c_char_p
        L.cdq_strerror.argtypes = [i32]
        L.cdq_workspace_bytes.restype = sz
        L.cdq_workspace_bytes.argtypes = [i32, i64, i64, i64]
        L.cdq_hessian.argtypes = [vp, i32, i64, i64, vp, i32, f32, vp, sz, vp]
        L.cdq_init_rtn.argtypes = [vp, i64, i64, i32, i64, vp, vp, vp, vp]
        L.cdq_gradient.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, vp, vp]
        L.cdq_greedy_cd.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, i64, i64, vp, vp, sz, vp]
        L.cdq_greedy_cd_ex.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, i64, i64, vp, ctypes.POINTER(CdOptions), vp, sz, vp]
        L.cdq_loss.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, vp, vp, vp, sz, vp]
        L.cdq_init_owc.argtypes = [vp, vp, i64, i64, i32, i64, i32, f32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.cdq_init_owc.restype = i32
        L.cdq_score_argmin.argtypes = [vp, vp, vp, vp, i64, i64, i32, i64, vp, vp, vp, vp]
        L.cdq_gather_update.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, vp, vp, vp]
        L.cdq_greedy_cd_stepwise.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, i64, i64, vp, vp, sz, vp]
        for fn in (L.cdq_score_argmin, L.cdq_gather_update, L.cdq_greedy_cd_stepwise):
            fn.restype = i32
        L.cdq_init_owc_cd.argtypes = [vp, vp, i64, i64, i32, i64, i32, i64, vp, vp, vp, vp, vp, vp, i64, i32, vp, sz, vp]
        L.cdq_init_owc_cd.restype = i32
        L.cdq_bcd.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, i64, i32, vp, i64, vp, vp, vp, i64, i32, vp, sz, vp]
        L.cdq_bcd.restype = i32
        L.cdq_cyclic_cd.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, i64, i64, vp, vp, vp, i64, vp, sz, vp]
        L.cdq_cyclic_cd.restype = i32
        L.cdq_loss_static.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, vp, vp, vp]
        L.cdq_loss_static.restype = i32
        L.cdq_greedy_cd_shape.argtypes = [i64, i64, i64, i32, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32),
                                          ctypes.POINTER(ctypes.c_int32)]
        L.cdq_greedy_cd_shape.restype = i32
        L.cdq_probe_mfma.argtypes = [i32, i64, i64, vp, ctypes.POINTER(ctypes.c_double), vp]
        L.cdq_probe_mfma.restype = i32
        L.cdq_probe_copy.argtypes = [vp, vp, sz, vp]
        L.cdq_probe_read.argtypes = [vp, sz, vp, vp]
        L.cdq_probe_gather.argtypes = [vp, i64, i64, i64, i32, i64, vp, vp]
        for fn in (L.cdq_hessian, L.cdq_init_rtn, L.cdq_gradient, L.cdq_greedy_cd, L.cdq_greedy_cd_ex, L.cdq_loss,
                   L.cdq_probe_copy, L.cdq_probe_read, L.cdq_probe_gather):
            fn.restype = i32
        _lib = L
    return _lib


def _check(code: int, what: str) -> None:
    if code != 0:
        raise CdqError(code, what)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype, what: str) -> int:
    if not (t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise TypeError(f"{what}: need a contiguous CUDA tensor of {dtype}, got {t.dtype} on {t.device}")
    return t.data_ptr()


def _out(t: torch.Tensor, dtype, shape, what: str) -> int:
    if tuple(t.shape) != tuple(shape):
        raise TypeError(f"{what}: need shape {tuple(shape)}, got {tuple(t.shape)}")
    return _dev(t, dtype, what)


def workspace_bytes(op: int, n: int, d_out: int, d_in: int) -> int:
    return int(lib().cdq_workspace_bytes(op, n, d_out, d_in))


def _workspace(op: int, n: int, d_out: int, d_in: int, ws: torch.Tensor | None) -> torch.Tensor:
    need = max(workspace_bytes(op, n, d_out, d_in), 256)
    if ws is None:
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    return ws


def hessian(X: torch.Tensor, H: torch.Tensor | None = None, accumulate: bool = False, lambda_rel: float = 0.0,
            workspace: torch.Tensor | None = None) -> torch.Tensor:
    """H = X^T X (+ damping).  X [n][d_in] bf16 or fp32 on the GPU."""
    n, d_in = X.shape
    if X.dtype == torch.bfloat16:
        dt = CDQ_BF16
    elif X.dtype == torch.float32:
        dt = CDQ_F32
    else:
        raise TypeError("X must be bfloat16 or float32")
    if H is None:
        if accumulate:
            raise ValueError("accumulate needs an existing H")
        H = torch.empty((d_in, d_in), dtype=torch.float32, device=X.device)
    ws = _workspace(OP_HESSIAN, n, 0, d_in, workspace)
    _check(lib().cdq_hessian(_dev(X, X.dtype, "X"), dt, n, d_in, _dev(H, torch.float32, "H"), int(accumulate),
                             float(lambda_rel), ws.data_ptr(), ws.numel(), _stream()), "cdq_hessian")
    return H


def init_rtn(Wt: torch.Tensor, bits: int, group: int):
    """MinMax grid + round-to-nearest codes.  Returns (scale, zero, Q)."""
    d_out, d_in = Wt.shape
    n_grp = d_in // group if group > 0 and d_in % group == 0 else 1
    scale = torch.empty((d_out, n_grp), dtype=torch.float32, device=Wt.device)
    zero = torch.empty((d_out, n_grp), dtype=torch.float32, device=Wt.device)
    Q = torch.empty((d_out, d_in), dtype=torch.uint8, device=Wt.device)
    _check(lib().cdq_init_rtn(_dev(Wt, torch.float32, "Wt"), d_out, d_in, bits, group, scale.data_ptr(), zero.data_ptr(),
                              Q.data_ptr(), _stream()), "cdq_init_rtn")
    return scale, zero, Q


def init_owc(H, Wt, bits: int, group: int, n_gamma: int = 50, workspace: torch.Tensor | None = None, want_loss: bool = True,
             screen_margin: float = 0.0, want_researched: bool = False, G_out: torch.Tensor | None = None):
    """OWC grid search (per-channel).  Returns (scale, zero, Q, gamma, loss_per_col); loss_per_col is None when
    want_loss is False.  With want_researched a sixth value: an int32 tensor [1], the number of columns whose fp16
    estimate failed its check and were searched exhaustively in fp64.  G_out: an fp32 [d_out][d_in] tensor that
    receives the gradient H e of the returned grid (to be handed to greedy_cd as G0)."""
    d_out, d_in = Wt.shape
    scale = torch.empty((d_out, 1), dtype=torch.float32, device=Wt.device)
    zero = torch.empty((d_out, 1), dtype=torch.float32, device=Wt.device)
    Q = torch.empty((d_out, d_in), dtype=torch.uint8, device=Wt.device)
    gamma = torch.empty(d_out, dtype=torch.float32, device=Wt.device)
    per = torch.empty(d_out, dtype=torch.float64, device=Wt.device) if want_loss else None
    cnt = torch.zeros(1, dtype=torch.int32, device=Wt.device) if want_researched else None
    ws = _workspace(OP_INIT_OWC, 0, d_out, d_in, workspace)
    _check(lib().cdq_init_owc(_dev(H, torch.float32, "H"), _dev(Wt, torch.float32, "Wt"), d_out, d_in, bits, group, n_gamma,
                              float(screen_margin), scale.data_ptr(), zero.data_ptr(), Q.data_ptr(), gamma.data_ptr(),
                              per.data_ptr() if want_loss else None, cnt.data_ptr() if want_researched else None,
                              _out(G_out, torch.float32, (d_out, d_in), "G_out") if G_out is not None else None,
                              ws.data_ptr(), ws.numel(), _stream()), "cdq_init_owc")
    if want_researched:
        return scale, zero, Q, gamma, per, cnt
    return scale, zero, Q, gamma, per


def init_owc_cd(H, Wt, bits: int, group: int, n_gamma: int = 50, T: int | None = None, trace_cap: int = 0,
                variant: int = 0, workspace: torch.Tensor | None = None):
    """OWC-CD (Algorithm 3) for sub-channel grids.  Returns a dict: scale, zero, Q, gamma_idx, moves[, trace]."""
    d_out, d_in = Wt.shape
    n_grp = d_in // group
    if T is None:
        T = n_grp
    dev_ = Wt.device
    out = {"scale": torch.empty((d_out, n_grp), dtype=torch.float32, device=dev_),
           "zero": torch.empty((d_out, n_grp), dtype=torch.float32, device=dev_),
           "Q": torch.empty((d_out, d_in), dtype=torch.uint8, device=dev_),
           "gamma_idx": torch.empty((d_out, n_grp), dtype=torch.int32, device=dev_),
           "moves": torch.zeros(d_out, dtype=torch.int32, device=dev_)}
    ws = _workspace(OP_INIT_OWC_CD, 0, d_out, d_in, workspace)
    tr = None
    if trace_cap > 0:
        out["trace"] = torch.full((d_out, trace_cap), -1, dtype=torch.int32, device=dev_)
        tr = out["trace"].data_ptr()
    _check(lib().cdq_init_owc_cd(_dev(H, torch.float32, "H"), _dev(Wt, torch.float32, "Wt"), d_out, d_in, bits, group, n_gamma, T,
                                 out["scale"].data_ptr(), out["zero"].data_ptr(), out["Q"].data_ptr(), out["gamma_idx"].data_ptr(),
                                 out["moves"].data_ptr(), tr, trace_cap, variant, ws.data_ptr(), ws.numel(), _stream()), "cdq_init_owc_cd")
    return out


def bcd(H, Wt, scale, zero, Q, bits: int, group: int, parts: torch.Tensor, k: int = 2, trace_cap: int = 0, want_G: bool = False,
        score_all: bool = False, single_column: bool = False, wide: bool = False, workspace: torch.Tensor | None = None):
    """Block coordinate descent with random blocks (Algorithm 2/5); Q is updated in place.  parts [T][d_in] int32 on
    the GPU.  score_all / single_column / wide set bits 0 / 1 / 2 of the entry point's flags (same results, for tests and timing).
    Returns a dict: moves[, trace [d_out][trace_cap][4]][, G]."""
    d_out, d_in = Wt.shape
    T = int(parts.shape[0])
    if parts.dtype != torch.int32 or not parts.is_cuda or not parts.is_contiguous() or (T and parts.shape[1] != d_in):
        raise TypeError("parts must be a contiguous int32 CUDA tensor [T][d_in]")
    ws = _workspace(OP_BCD, T, d_out, d_in, workspace)
    out = {"moves": torch.zeros(d_out, dtype=torch.int32, device=Wt.device)}
    tr = g = None
    if trace_cap > 0:
        out["trace"] = torch.full((d_out, trace_cap, 4), -1, dtype=torch.int32, device=Wt.device)
        tr = out["trace"].data_ptr()
    if want_G:
        out["G"] = torch.empty((d_out, d_in), dtype=torch.float32, device=Wt.device)
        g = out["G"].data_ptr()
    _check(lib().cdq_bcd(_dev(H, torch.float32, "H"), _dev(Wt, torch.float32, "Wt"), _dev(scale, torch.float32, "scale"),
                         _dev(zero, torch.float32, "zero"), _dev(Q, torch.uint8, "Q"), d_out, d_in, bits, group, k,
                         parts.data_ptr() if T else None, T, out["moves"].data_ptr(), g, tr, trace_cap, int(score_all) | (2 if single_column else 0) | (4 if wide else 0),
                         ws.data_ptr(), ws.numel(), _stream()), "cdq_bcd")
    return out


def cyclic_cd(H, Wt, scale, zero, Q, bits: int, group: int, T: int, trace_cap: int = 0, want_G: bool = False,
              workspace: torch.Tensor | None = None):
    """Cyclic coordinate descent in place on Q; T visits at most.  Returns a dict: stats (int32 [d_out][4] view:
    moves, iters, converged, bits of the last score)[, trace][, G]."""
    d_out, d_in = Wt.shape
    ws = _workspace(OP_CYCLIC_CD, 0, d_out, d_in, workspace)
    out = {"stats": torch.zeros((d_out, 4), dtype=torch.int32, device=Wt.device)}
    tr = g = None
    if trace_cap > 0:
        out["trace"] = torch.full((d_out, trace_cap), -1, dtype=torch.int32, device=Wt.device)
        tr = out["trace"].data_ptr()
    if want_G:
        out["G"] = torch.empty((d_out, d_in), dtype=torch.float32, device=Wt.device)
        g = out["G"].data_ptr()
    _check(lib().cdq_cyclic_cd(_dev(H, torch.float32, "H"), _dev(Wt, torch.float32, "Wt"), _dev(scale, torch.float32, "scale"),
                               _dev(zero, torch.float32, "zero"), _dev(Q, torch.uint8, "Q"), d_out, d_in, bits, group, T,
                               out["stats"].data_ptr(), g, tr, trace_cap, ws.data_ptr(), ws.numel(), _stream()), "cdq_cyclic_cd")
    return out


def gradient(H, Wt, scale, zero, Q, group: int) -> torch.Tensor:
    """G = E H, E = scale*Q + zero - Wt (fp64 accumulation, fp32 result)."""
    d_out, d_in = Wt.shape
    G = torch.empty((d_out, d_in), dtype=torch.float32, device=Wt.device)
    _check(lib().cdq_gradient(_dev(H, torch.float32, "H"), _dev(Wt, torch.float32, "Wt"), _dev(scale, torch.float32, "scale"),
                              _dev(zero, torch.float32, "zero"), _dev(Q, torch.uint8, "Q"), d_out, d_in, group,
                              G.data_ptr(), _stream()), "cdq_gradient")
    return G


def greedy_cd(H, Wt, scale, zero, Q, bits: int, group: int, T: int, stats: bool = True,
              workspace: torch.Tensor | None = None, waves_per_column: int = 0, elems_per_lane: int = 0,
              trace_cap: int = 0, want_G: bool = False, loop_events=None, exact_scorer_only: bool = False,
              G0: torch.Tensor | None = None, teams_per_cu: int = 0):
    """Greedy coordinate descent in place on Q.  Returns a dict with 'stats' (int32 [d_out][4] view:
    moves, iters, converged, last_score bits), and optionally 'trace' and 'G'.  loop_events is an
    optional pair of raw hipEvent_t handles recorded around the iteration-loop kernel.  G0: the start gradient
    of (scale, zero, Q) from gradient() or init_owc(G_out=...); it is consumed (overwritten) and the gradient
    initialisation is skipped."""
    d_out, d_in = Wt.shape
    if G0 is None:
        ws = _workspace(OP_GREEDY_CD, 0, d_out, d_in, workspace)
    elif workspace is not None:
        ws = workspace
    else:
        ws = torch.empty((4 * d_in + 255) // 256 * 256, dtype=torch.uint8, device=Wt.device)
    st = torch.zeros((d_out, 4), dtype=torch.int32, device=Wt.device) if stats else None
    out = {}
    opts = CdOptions(waves_per_column, elems_per_lane, int(exact_scorer_only), int(teams_per_cu), None, 0, None, None, None, None)
    if G0 is not None:
        opts.G0 = _out(G0, torch.float32, (d_out, d_in), "G0")
    if loop_events is not None:            # (begin, end) raw hipEvent_t handles
        opts.ev_loop_begin, opts.ev_loop_end = loop_events
    if trace_cap > 0:
        out["trace"] = torch.full((d_out, trace_cap), -1, dtype=torch.int32, device=Wt.device)
        opts.trace = out["trace"].data_ptr()
        opts.trace_cap = trace_cap
    if want_G:
        out["G"] = torch.empty((d_out, d_in), dtype=torch.float32, device=Wt.device)
        opts.G_out = out["G"].data_ptr()
    _check(lib().cdq_greedy_cd_ex(_dev(H, torch.float32, "H"), _dev(Wt, torch.float32, "Wt"),
                                  _dev(scale, torch.float32, "scale"), _dev(zero, torch.float32, "zero"),
                                  _dev(Q, torch.uint8, "Q"), d_out, d_in, bits, group, T,
                                  st.data_ptr() if st is not None else None, ctypes.byref(opts),
                                  ws.data_ptr(), ws.numel(), _stream()), "cdq_greedy_cd")
    out["stats"] = st
    return out


def greedy_cd_shape(d_out: int, d_in: int, group: int, aligned16: bool = True):
    """(wavefronts per column, coordinates per lane) that greedy_cd takes for a layer by default."""
    return greedy_cd_launch(d_out, d_in, group, aligned16)[:2]


def greedy_cd_launch(d_out: int, d_in: int, group: int, aligned16: bool = True):
    """(wavefronts per column, coordinates per lane, columns resident per compute unit) of greedy_cd's default launch."""
    w, e, t = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_int32(0)
    _check(lib().cdq_greedy_cd_shape(d_out, d_in, group, int(aligned16), ctypes.byref(w), ctypes.byref(e), ctypes.byref(t)),
           "cdq_greedy_cd_shape")
    return int(w.value), int(e.value), int(t.value)


def score_argmin(Hdiag, scale, Q, G, bits: int, group: int):
    """Arg-min step of one iteration.  Returns (best_i int32, best_r int32, best_s fp32), each [d_out]."""
    d_out, d_in = Q.shape
    bi = torch.empty(d_out, dtype=torch.int32, device=Q.device)
    br = torch.empty(d_out, dtype=torch.int32, device=Q.device)
    bs = torch.empty(d_out, dtype=torch.float32, device=Q.device)
    _check(lib().cdq_score_argmin(_dev(Hdiag, torch.float32, "Hdiag"), _dev(scale, torch.float32, "scale"), _dev(Q, torch.uint8, "Q"),
                                  _dev(G, torch.float32, "G"), d_out, d_in, bits, group, bi.data_ptr(), br.data_ptr(),
                                  bs.data_ptr(), _stream()), "cdq_score_argmin")
    return bi, br, bs


def gather_update(H, scale, Q, G, group: int, best_i, best_r, moves=None) -> None:
    """Code and gradient update of one iteration, in place on Q and G."""
    d_out, d_in = Q.shape
    _check(lib().cdq_gather_update(_dev(H, torch.float32, "H"), _dev(scale, torch.float32, "scale"), _dev(Q, torch.uint8, "Q"),
                                   _dev(G, torch.float32, "G"), d_out, d_in, group, _dev(best_i, torch.int32, "best_i"),
                                   _dev(best_r, torch.int32, "best_r"), moves.data_ptr() if moves is not None else None,
                                   _stream()), "cdq_gather_update")


def greedy_cd_stepwise(H, Wt, scale, zero, Q, bits: int, group: int, T: int, workspace: torch.Tensor | None = None):
    """Greedy CD as 2T separate launches (general path, any d_in).  Returns per-column move counts."""
    d_out, d_in = Wt.shape
    ws = _workspace(OP_GREEDY_CD, 0, d_out, d_in, workspace)
    moves = torch.zeros(d_out, dtype=torch.int32, device=Wt.device)
    _check(lib().cdq_greedy_cd_stepwise(_dev(H, torch.float32, "H"), _dev(Wt, torch.float32, "Wt"), _dev(scale, torch.float32, "scale"),
                                        _dev(zero, torch.float32, "zero"), _dev(Q, torch.uint8, "Q"), d_out, d_in, bits, group, T,
                                        moves.data_ptr(), ws.data_ptr(), ws.numel(), _stream()), "cdq_greedy_cd_stepwise")
    return moves


def loss(H, Wt, scale, zero, Q, group: int, workspace: torch.Tensor | None = None):
    """Returns (loss_per_col fp64 [d_out], loss_total fp64 [1]) as device tensors."""
    d_out, d_in = Wt.shape
    ws = _workspace(OP_LOSS, 0, d_out, d_in, workspace)
    per = torch.empty(d_out, dtype=torch.float64, device=Wt.device)
    tot = torch.empty(1, dtype=torch.float64, device=Wt.device)
    _check(lib().cdq_loss(_dev(H, torch.float32, "H"), _dev(Wt, torch.float32, "Wt"), _dev(scale, torch.float32, "scale"),
                          _dev(zero, torch.float32, "zero"), _dev(Q, torch.uint8, "Q"), d_out, d_in, group,
                          per.data_ptr(), tot.data_ptr(), ws.data_ptr(), ws.numel(), _stream()), "cdq_loss")
    return per, tot


def loss_static(H, Wt, scale, zero, Q, group: int, per: torch.Tensor, tot: torch.Tensor) -> None:
    """cdq_loss_static: the loss with the partial sums in the library's own static device array.  The call allocates
    nothing, so the caller passes the outputs: per [d_out] fp64, tot [1] fp64."""
    d_out, d_in = Wt.shape
    _check(lib().cdq_loss_static(_dev(H, torch.float32, "H"), _dev(Wt, torch.float32, "Wt"), _dev(scale, torch.float32, "scale"),
                                 _dev(zero, torch.float32, "zero"), _dev(Q, torch.uint8, "Q"), d_out, d_in, group,
                                 _dev(per, torch.float64, "per"), _dev(tot, torch.float64, "tot"), _stream()), "cdq_loss_static")


# ---- measurement helpers (see include/cdq.h): thin wrappers, used by bench.py only

def probe_copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    nbytes = src.numel() * src.element_size()
    _check(lib().cdq_probe_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream()), "cdq_probe_copy")


def probe_read(src: torch.Tensor, nbytes: int, sink: torch.Tensor) -> None:
    _check(lib().cdq_probe_read(src.data_ptr(), nbytes, sink.data_ptr(), _stream()), "cdq_probe_read")


def probe_gather(H: torch.Tensor, n_rows: int, row_bytes: int, teams: int, waves_per_row: int, iters: int,
                 sink: torch.Tensor) -> None:
    _check(lib().cdq_probe_gather(H.data_ptr(), n_rows, row_bytes, teams, waves_per_row, iters, sink.data_ptr(),
                                  _stream()), "cdq_probe_gather")


def probe_mfma(kind: int, blocks: int, iters: int, sink: torch.Tensor) -> float:
    """Launches the matrix-core-only loop (kind 0: bf16 32x32x16, 1: fp64 16x16x4); returns its operation count."""
    flop = ctypes.c_double(0.0)
    _check(lib().cdq_probe_mfma(kind, blocks, iters, sink.data_ptr(), ctypes.byref(flop), _stream()), "cdq_probe_mfma")
    return float(flop.value)
