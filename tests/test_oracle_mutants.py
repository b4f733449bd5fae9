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
