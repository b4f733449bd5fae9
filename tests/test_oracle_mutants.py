"""The pins must be able to fail: plant one plausible mistake at a time in a private copy
of the oracle's C source (on the CPU), and check that a pin catches it -- the committed
scores no longer equal the loss change recomputed from X, or the end point is no longer a
coordinate-wise optimum."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

from oracle import paper_form as pf

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "cdq_oracle.c")

MUTANTS = {
    "dropped_factor_2": ("const float two_g = 2.0f * g[i];", "const float two_g = g[i];"),
    "wrong_sign_update": ("g[k] = fmaf(delta, hrow[k], g[k]);", "g[k] = fmaf(-delta, hrow[k], g[k]);"),
    "dropped_quadratic_term": ("const float s = delta * fmaf(delta, hii, two_g);\n                    if (s < best_s) { best_s = s; best_i = i; best_r = r; }",
                               "const float s = delta * two_g;\n                    if (s < best_s) { best_s = s; best_i = i; best_r = r; }"),
    "wrong_row_index": ("const float *hrow = H + best_i * d_in;         /* H symmetric: row = column */",
                        "const float *hrow = H + best_r * d_in;"),
    "scale_of_wrong_group": ("const float ai = a[i / group];\n                const float hii = H[i * d_in + i];\n                const float two_g",
                             "const float ai = a[0];\n                const float hii = H[i * d_in + i];\n                const float two_g"),
    "residual_sign": ("E[j * d_in + i] = fmaf(a, (float)Q[j * d_in + i], b) - Wt[j * d_in + i];",
                      "E[j * d_in + i] = Wt[j * d_in + i] - fmaf(a, (float)Q[j * d_in + i], b);"),
}


def _pins_hold(lib):
    """Run fp32 CD through `lib` on a small correlated group-wise layer and apply two pins."""
    rng = np.random.default_rng(3)
    d_in, d_out, n, bits, group = 16, 4, 64, 3, 4
    X = rng.standard_normal((n, d_in)) + rng.standard_normal((n, 1))
    Wt = (rng.standard_normal((d_out, d_in)) / 4).astype(np.float32)
    H = (X.T @ X).astype(np.float32)
    Wg = Wt.reshape(d_out, d_in // group, group)
    b = Wg.min(2).astype(np.float32)
    a = ((Wg.max(2) - b) / np.float32(7)).astype(np.float32)
    q = rng.integers(0, 8, (d_out, d_in)).astype(np.uint8)
    q0 = q.copy()
    p = lambda x: x.ctypes.data_as(ctypes.c_void_p)
    I = ctypes.c_int64
    E = np.empty((d_out, d_in), np.float32)
    lib.cdqo_residual_f32(p(Wt), p(q), p(a), p(b), I(d_out), I(d_in), I(group), p(E))
    G = np.empty_like(E)
    lib.cdqo_gradient_f32(p(H), p(E), I(d_out), I(d_in), p(G))
    cap = 4 * d_in
    mv = np.zeros(d_out, np.int32); cv = np.zeros(d_out, np.int32)
    ti = np.zeros((d_out, cap), np.int32); tr = np.zeros((d_out, cap), np.int32); ts = np.zeros((d_out, cap), np.float32)
    lib.cdqo_greedy_cd_f32(p(H), p(a), p(q), p(G), I(d_out), I(d_in), ctypes.c_int(bits), I(group), I(cap),
                           p(mv), p(cv), p(ti), p(tr), p(ts), I(cap))
    ok = True
    for j in range(d_out):
        av = np.repeat(a[j].astype(np.float64), group); bv = np.repeat(b[j].astype(np.float64), group)
        w = Wt[j].astype(np.float64)
        cur = q0[j].astype(np.float64)
        prev = pf.layer_loss(X, w, av, bv, cur)
        for k in range(mv[j]):
            cur[ti[j, k]] = tr[j, k]
            now = pf.layer_loss(X, w, av, bv, cur)
            ok &= abs((now - prev) - ts[j, k]) <= 1e-3 * max(abs(prev), 1.0)
            prev = now
        ok &= bool(cv[j] == 1)
        for i in range(d_in):                      # coordinate-wise optimum
            for lev in range(8):
                alt = q[j].astype(np.float64); alt[i] = lev
                ok &= pf.layer_loss(X, w, av, bv, alt) >= prev * (1 - 1e-5)
    return bool(ok)


OWC_CD_MUTANTS = {
    "v_sign_as_printed": ("            v[r] = 2.0 * acc;", "            v[r] = -2.0 * acc;"),
    "v_update_factor": ("                v[r] += 2.0 * acc;", "                v[r] += acc;"),
    "v_update_wrong_block": ("const float *hrow = H + r * d_in + best_i * group;", "const float *hrow = H + r * d_in;"),
    "quadratic_term_doubled": ("s += d[m] * (row + v[i * group + m]);", "s += d[m] * (2.0 * row + v[i * group + m]);"),
    "residual_not_committed": ("for (int64_t m = 0; m < group; ++m) e[best_i * group + m] = en[m];", ""),
}


def _owc_cd_pins_hold(lib):
    """Algorithm 3 through `lib` on a small layer: every committed score is the loss change recomputed
    from X, and at a converged end point no single group can lower the loss by another grid point."""
    rng = np.random.default_rng(5)
    d_in, d_out, n, bits, group, n_gamma = 24, 3, 80, 2, 6, 10
    X = rng.standard_normal((n, d_in)) + 0.5 * rng.standard_normal((n, 1))
    Wt = (rng.standard_normal((d_out, d_in)) / 4).astype(np.float32)
    Wt[:, ::7] *= 4.0
    H = (X.T @ X).astype(np.float32)
    n_grp, T = d_in // group, 40
    p = lambda x: x.ctypes.data_as(ctypes.c_void_p)
    I = ctypes.c_int64
    scale = np.empty((d_out, n_grp), np.float32); zero = np.empty_like(scale)
    Q = np.empty((d_out, d_in), np.uint8); gi = np.zeros((d_out, n_grp), np.int32)
    mv = np.zeros(d_out, np.int32); cv = np.zeros(d_out, np.int32)
    ti = np.full((d_out, T), -1, np.int32); tr = np.full((d_out, T), -1, np.int32); ts = np.zeros((d_out, T))
    lib.cdqo_owc_cd(p(H), p(Wt), I(d_out), I(d_in), ctypes.c_int(bits), I(group), ctypes.c_int(n_gamma), I(T),
                    p(scale), p(zero), p(Q), p(gi), p(mv), p(cv), p(ti), p(tr), p(ts), I(T))
    H64 = H.astype(np.float64)

    def loss_of(j, ks):
        e = np.empty(d_in)
        for i in range(n_grp):
            sl = slice(i * group, (i + 1) * group)
            w = Wt[j, sl]
            a = np.float32(np.float32(np.float32(ks[i]) / np.float32(n_gamma)) * (w.max() - w.min())) / np.float32(3)
            a = a if a > 0 else np.float32(1)
            q = np.clip(np.rint((w - w.min()) / a), 0, 3).astype(np.float32)
            e[sl] = (a * q + w.min()).astype(np.float32) - w
        return float(e @ H64 @ e)

    ok = True
    for j in range(d_out):
        ks = [n_gamma] * n_grp
        prev = loss_of(j, ks)
        for m in range(mv[j]):
            ks[ti[j, m]] = tr[j, m]
            now = loss_of(j, ks)
            ok &= abs((now - prev) - ts[j, m]) <= 1e-4 * max(abs(prev), 1e-9)
            prev = now
        ok &= list(gi[j]) == ks
        if cv[j]:
            for i in range(n_grp):
                for k in range(1, n_gamma + 1):
                    alt = list(ks); alt[i] = k
                    ok &= loss_of(j, alt) >= prev * (1 - 1e-6)
    return bool(ok) and bool(mv.sum() > 0)


BCD_MUTANTS = {
    "cross_term_factor": ("s = fmaf(delta[m] * delta[m2], 2.0f * H[(int64_t)mem[m] * d_in + mem[m2]], s);",
                          "s = fmaf(delta[m] * delta[m2], H[(int64_t)mem[m] * d_in + mem[m2]], s);"),
    "cross_term_wrong_entry": ("s = fmaf(delta[m] * delta[m2], 2.0f * H[(int64_t)mem[m] * d_in + mem[m2]], s);",
                               "s = fmaf(delta[m] * delta[m2], 2.0f * H[(int64_t)mem[m] * d_in + mem[m]], s);"),
    "committed_block_offset": ("const int32_t *mem = part + best_b * k;\n            int64_t rest = best_tuple;",
                               "const int32_t *mem = part + best_b;\n            int64_t rest = best_tuple;"),
    "update_with_wrong_member_level": ("const float delta = a[c / group] * (float)(r_new[m] - (int)q[c]);",
                                       "const float delta = a[c / group] * (float)(r_new[0] - (int)q[c]);"),
    "gradient_update_sign": ("for (int64_t x = 0; x < d_in; ++x) g[x] = fmaf(delta, hrow[x], g[x]);",
                             "for (int64_t x = 0; x < d_in; ++x) g[x] = fmaf(-delta, hrow[x], g[x]);"),
}


def _bcd_pins_hold(lib):
    """Algorithm 2 (k = 2) through `lib`: committed scores are loss changes, and an iteration without a move
    leaves no block of its partition improvable."""
    import itertools
    rng = np.random.default_rng(12)
    d_in, d_out, n, bits, group, k, T = 8, 3, 50, 2, 4, 2, 16
    X = rng.standard_normal((n, d_in)) + 0.7 * rng.standard_normal((n, 1))
    Wt = (rng.standard_normal((d_out, d_in)) / 3).astype(np.float32)
    H = (X.T @ X).astype(np.float32)
    Wg = Wt.reshape(d_out, d_in // group, group)
    b = Wg.min(2).astype(np.float32)
    a = ((Wg.max(2) - b) / np.float32(3)).astype(np.float32)
    q = rng.integers(0, 4, (d_out, d_in)).astype(np.uint8)
    q0 = q.copy()
    parts = np.stack([rng.permutation(d_in) for _ in range(T)]).astype(np.int32)
    p = lambda x: x.ctypes.data_as(ctypes.c_void_p)
    I = ctypes.c_int64
    E = np.empty((d_out, d_in), np.float32)
    lib.cdqo_residual_f32(p(Wt), p(q), p(a), p(b), I(d_out), I(d_in), I(group), p(E))
    G = np.empty_like(E)
    lib.cdqo_gradient_f32(p(H), p(E), I(d_out), I(d_in), p(G))
    mv = np.zeros(d_out, np.int32)
    tt, tb, tr = (np.full((d_out, T), -1, np.int32) for _ in range(3))
    ts = np.zeros((d_out, T), np.float32)
    lib.cdqo_bcd_f32(p(H), p(a), p(q), p(G), p(parts), I(d_out), I(d_in), ctypes.c_int(bits), I(group), ctypes.c_int(k), I(T),
                     p(mv), p(tt), p(tb), p(tr), p(ts), I(T))
    ok = bool(mv.sum() > 0)
    for j in range(d_out):
        av = np.repeat(a[j].astype(np.float64), group); bv = np.repeat(b[j].astype(np.float64), group)
        w = Wt[j].astype(np.float64)
        cur = q0[j].astype(np.float64)
        prev = pf.layer_loss(X, w, av, bv, cur)
        moved = {int(t): m for m, t in enumerate(tt[j]) if t >= 0}
        for t in range(T):
            if t in moved:
                m = moved[t]
                blk = parts[t, k * tb[j, m]: k * tb[j, m] + k]
                for mm, c in enumerate(blk):
                    cur[c] = (tr[j, m] >> (4 * mm)) & 15
                now = pf.layer_loss(X, w, av, bv, cur)
                ok &= abs((now - prev) - ts[j, m]) <= 1e-3 * max(abs(prev), 1.0)
                prev = now
            else:
                for bi in range(d_in // k):
                    blk = parts[t, k * bi: k * bi + k]
                    for tup in itertools.product(range(4), repeat=k):
                        alt = cur.copy(); alt[blk] = tup
                        ok &= pf.layer_loss(X, w, av, bv, alt) >= prev * (1 - 1e-5)
        ok &= np.array_equal(cur.astype(np.uint8), q[j])
    return bool(ok)


def _compile(src_text, tmp_path, name):
    c = tmp_path / f"{name}.c"
    so = tmp_path / f"{name}.so"
    c.write_text(src_text)
    subprocess.run(["gcc", "-O1", "-std=c99", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", str(c), "-o", str(so), "-lm"],
                   check=True)
    return ctypes.CDLL(str(so))


def test_unmutated_source_passes(tmp_path):
    assert _pins_hold(_compile(open(SRC).read(), tmp_path, "orig"))


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pin_catches_mutant(tmp_path, name):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) >= 1, "mutation site not found: the oracle source changed, update this test"
    assert not _pins_hold(_compile(text.replace(old, new, 1), tmp_path, name))


def test_unmutated_source_passes_owc_cd_pins(tmp_path):
    assert _owc_cd_pins_hold(_compile(open(SRC).read(), tmp_path, "orig_owc"))


@pytest.mark.parametrize("name", sorted(OWC_CD_MUTANTS))
def test_owc_cd_pin_catches_mutant(tmp_path, name):
    old, new = OWC_CD_MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) == 1, "mutation site not found: the oracle source changed, update this test"
    assert not _owc_cd_pins_hold(_compile(text.replace(old, new, 1), tmp_path, name))


def test_unmutated_source_passes_bcd_pins(tmp_path):
    assert _bcd_pins_hold(_compile(open(SRC).read(), tmp_path, "orig_bcd"))


@pytest.mark.parametrize("name", sorted(BCD_MUTANTS))
def test_bcd_pin_catches_mutant(tmp_path, name):
    old, new = BCD_MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) == 1, "mutation site not found: the oracle source changed, update this test"
    assert not _bcd_pins_hold(_compile(text.replace(old, new, 1), tmp_path, name))
