"""GPU parity: every stage of the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Bars:
  init_rtn          bit-exact
  hessian           |dH_ik| <= 8 sqrt(n) 2^-24 sqrt(H_ii H_kk) and relative Frobenius error <= 1e-5
  gradient          equal to the oracle's correctly-rounded fp32 value except at fp64 rounding
                    boundaries (<= 1e-6 of entries, each within 1 ulp)
  greedy_cd         fed the same fp32 H: codes equal on >= 99.9 % of entries; every column that
                    differs must diverge at a score tie; final loss within 1e-4 relative
  loss              within 1e-6 relative of the oracle's fp64 value (the kernel rounds e to fp32
                    first; given that fp32 e it matches an fp64 evaluation to 1e-12)
"""
import time

import numpy as np
import pytest
import torch

from paper_2406_17542_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def cdq():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2406_17542_amd import cdq as m
    m.lib()
    return m


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def x_to_dev(X, x_dtype):
    if x_dtype == "bf16":
        return dev(inputs.bf16_bits(X).view(np.int16)).view(torch.bfloat16)
    return dev(X.astype(np.float32))


def rand_layer(seed, d_in, d_out, n, corr=1.0):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, d_in)).astype(np.float32)
    if corr:
        X += (corr * rng.standard_normal((n, 1))).astype(np.float32)
    Wt = (rng.standard_normal((d_out, d_in)) / np.sqrt(d_in)).astype(np.float32)
    return X, Wt


def hessian_tolerance_ok(H_gpu, H64, n):
    d = np.sqrt(np.diag(H64))
    bound = 8.0 * np.sqrt(n) * 2.0 ** -24 * np.outer(d, d) + 1e-30
    err = np.abs(H_gpu.astype(np.float64) - H64)
    fro = np.linalg.norm(err) / max(np.linalg.norm(H64), 1e-300)
    return bool((err <= bound).all()), float((err / bound).max()), float(fro)


# ----------------------------------------------------------------------------- init_rtn

@pytest.mark.parametrize("d_out,d_in,bits,group", [
    (64, 128, 4, 128), (7, 96, 3, 32), (5, 130, 2, 26), (3, 1000, 4, 1000), (33, 256, 2, 128), (2, 5, 3, 5), (4, 64, 3, 1),
])
def test_init_rtn_bit_exact(cdq, oracle, d_out, d_in, bits, group):
    rng = np.random.default_rng(d_in + bits)
    Wt = (rng.standard_normal((d_out, d_in)) / np.sqrt(d_in)).astype(np.float32)
    Wt[0, : min(d_in, group)] = 0.25                 # a constant group
    if d_in >= 6 and group >= 6:                     # exact halves: round-half-even must agree
        Wt[1, :6] = np.array([0.0, 0.5, 1.5, 2.5, 3.0, 1.0], np.float32) if bits == 2 else Wt[1, :6]
    a, b, q = oracle.init_grid(Wt, bits, group)
    s, z, Q = cdq.init_rtn(dev(Wt), bits, group)
    assert np.array_equal(s.cpu().numpy(), a)
    assert np.array_equal(z.cpu().numpy(), b)
    assert np.array_equal(Q.cpu().numpy(), q)


def test_init_rtn_tiny_config(cdq, oracle):
    cfg = inputs.CONFIGS["tiny"]
    _, Wt = inputs.make_layer(cfg)
    a, b, q = oracle.init_grid(Wt, cfg.bits, cfg.group)
    s, z, Q = cdq.init_rtn(dev(Wt), cfg.bits, cfg.group)
    assert np.array_equal(s.cpu().numpy(), a) and np.array_equal(z.cpu().numpy(), b) and np.array_equal(Q.cpu().numpy(), q)


# ----------------------------------------------------------------------------- hessian

@pytest.mark.parametrize("x_dtype,n,d_in", [
    ("f32", 512, 128), ("f32", 300, 132), ("f32", 1, 4), ("f32", 1000, 260),
    ("bf16", 512, 128), ("bf16", 333, 136), ("bf16", 4096, 392), ("bf16", 7, 8), ("bf16", 2500, 1024),
    # interior 256-wide tiles with 1, 2, 3, 4 and 5 steps of 32 tokens: every length of the load pipeline's start-up
    ("bf16", 32, 256), ("bf16", 64, 512), ("bf16", 96, 256), ("bf16", 128, 512), ("bf16", 160, 256), ("bf16", 1056, 768),
    # 23 and more tiles per side: the tile list is shared out over the XCDs, whole tiles go straight into H and every
    # share's leftover tiles are cut into token slices (ragged width and token count; slices long enough for the pipelined
    # loop; a single token)
    ("bf16", 200, 5896), ("bf16", 4096, 6144), ("bf16", 1, 6144),
])
def test_hessian(cdq, oracle, x_dtype, n, d_in):
    X = inputs.make_x("outlier8x20", n, d_in, seed=n, x_dtype=x_dtype)
    H64 = oracle.hessian(X)
    H = cdq.hessian(x_to_dev(X, x_dtype)).cpu().numpy()
    assert np.array_equal(H, H.T), "H must be exactly symmetric"
    ok, worst, fro = hessian_tolerance_ok(H, H64, n)
    assert ok and fro <= 1e-5, (worst, fro)


def test_hessian_tiny_config_and_repeatable(cdq, oracle):
    cfg = inputs.CONFIGS["tiny"]
    X, _ = inputs.make_layer(cfg)
    Xd = x_to_dev(X, cfg.x_dtype)
    H1 = cdq.hessian(Xd).cpu().numpy()
    H2 = cdq.hessian(Xd).cpu().numpy()
    assert np.array_equal(H1, H2)
    ok, worst, fro = hessian_tolerance_ok(H1, oracle.hessian(X), cfg.n)
    assert ok and fro <= 1e-5, (worst, fro)


def test_hessian_accumulate_and_damping(cdq, oracle):
    X = inputs.make_x("student_t4", 1536, 264, seed=3, x_dtype="bf16")
    Xd = x_to_dev(X, "bf16")
    H = cdq.hessian(Xd[:512].contiguous())
    H = cdq.hessian(Xd[512:1024].contiguous(), H=H, accumulate=True)
    H = cdq.hessian(Xd[1024:].contiguous(), H=H, accumulate=True, lambda_rel=0.01)
    Hn = H.cpu().numpy()
    H64 = oracle.hessian(X, lambda_rel=0.01)
    assert np.array_equal(Hn, Hn.T)
    ok, worst, fro = hessian_tolerance_ok(Hn, H64, 1536)
    assert ok and fro <= 1e-5, (worst, fro)
    # the damping really is there: compare the diagonal against the undamped oracle
    lam = 0.01 * np.mean(np.diag(oracle.hessian(X)))
    np.testing.assert_allclose(np.diag(Hn) - np.diag(oracle.hessian(X)), lam, rtol=1e-3)


def test_hessian_accumulate_on_wide_layers(cdq, oracle):
    """Streaming over token chunks where the tiles are shared out over the XCDs: whole tiles add to H in place, sliced tiles
    through the partial sums; chunks of different lengths, the last one with damping."""
    d_in = 6152
    X = inputs.make_x("lognormal_scales", 1000, d_in, seed=5, x_dtype="bf16")
    Xd = x_to_dev(X, "bf16")
    H = cdq.hessian(Xd[:512].contiguous())
    H = cdq.hessian(Xd[512:520].contiguous(), H=H, accumulate=True)
    H = cdq.hessian(Xd[520:].contiguous(), H=H, accumulate=True, lambda_rel=0.02)
    Hn = H.cpu().numpy()
    assert np.array_equal(Hn, Hn.T)
    ok, worst, fro = hessian_tolerance_ok(Hn, oracle.hessian(X, lambda_rel=0.02), 1000)
    assert ok and fro <= 1e-5, (worst, fro)
    # the same call twice gives the same bits (the slices are added in a fixed order)
    H2 = cdq.hessian(Xd[:512].contiguous())
    H2 = cdq.hessian(Xd[512:520].contiguous(), H=H2, accumulate=True)
    H2 = cdq.hessian(Xd[520:].contiguous(), H=H2, accumulate=True, lambda_rel=0.02)
    assert torch.equal(H, H2)


def layer_with_exact_ties(seed=0, d_in=256, d_out=4, n=2000):
    """Every weight on a grid point of Eq. (2) (scale 21/16, zero 0, 3 bits) except one per column, which sits exactly half
    way between two levels on a coordinate whose (21/16) H_ii rounds up in fp32 by less than a quarter of a unit in the
    last place.  Moving that coordinate up or down leaves the loss unchanged, and in fp32 both moves compute to a tiny
    negative score: Algorithm 1 alternates between them until its budget is spent."""
    from fractions import Fraction
    r = np.random.default_rng(seed)
    X = r.standard_normal((n, d_in)).astype(np.float32)
    H32 = np.ascontiguousarray(np.float32(X.astype(np.float64).T @ X.astype(np.float64)))
    good = []
    for i in range(2, d_in):
        p = Fraction(21, 16) * Fraction(float(H32[i, i]))
        f32 = np.float32(float(p))
        if 0 < Fraction(float(f32)) - p < Fraction(float(np.spacing(f32))) / 4:
            good.append(i)
    Wt = (np.float32(1.3125) * r.integers(0, 8, (d_out, d_in))).astype(np.float32)
    Wt[:, 0], Wt[:, 1] = 0.0, 9.1875
    for j in range(d_out):
        Wt[j, good[j]] = 3.28125
    return H32, Wt, good[:d_out]


@pytest.mark.parametrize("waves,elems,teams", [(0, 0, 0), (1, 8, 0), (1, 16, 0), (2, 16, 0), (4, 8, 0), (16, 4, 0), (16, 16, 1), (16, 16, 2),
                                               (16, 24, 0), (16, 32, 0), (16, 36, 0)])
def test_greedy_cd_alternating_between_two_levels_of_equal_loss(cdq, oracle, waves, elems, teams):
    """The kernels for 16-byte chunks jump over the rest of the budget once the state repeats; the oracle takes every step.
    Same moves, same codes, for even and odd budgets, and the same trajectory when it is traced (tracing switches the jump
    off)."""
    H32, Wt, ties = layer_with_exact_ties()
    d_out, d_in = Wt.shape
    a, b, q0 = oracle.init_grid(Wt, 3, d_in)
    assert np.all(a == np.float32(1.3125)) and np.all(b == 0)
    for T in (1, 2, 3, 50, 51, 400):
        ref = oracle.greedy_cd(H32, Wt, a, b, q0, 3, d_in, T)
        assert np.all(ref["moves"] == T), "the case should alternate to the end of every budget"
        Q = dev(q0.copy())
        out = cdq.greedy_cd(dev(H32), dev(Wt), dev(a), dev(b), Q, 3, d_in, T, waves_per_column=waves, elems_per_lane=elems, want_G=True,
                            teams_per_cu=teams)
        st = out["stats"].cpu().numpy()
        assert np.array_equal(st[:, 0], ref["moves"]) and np.all(st[:, 2] == 0), (T, st)
        assert np.array_equal(Q.cpu().numpy(), ref["Q"]), T
        assert np.array_equal(out["G"].cpu().numpy(), ref["G"]), T
        assert [int(Q.cpu().numpy()[j, i]) for j, i in enumerate(ties)] == [2 + T % 2] * d_out
    ref = oracle.greedy_cd(H32, Wt, a, b, q0, 3, d_in, 60, trace_cap=60)
    Q = dev(q0.copy())
    out = cdq.greedy_cd(dev(H32), dev(Wt), dev(a), dev(b), Q, 3, d_in, 60, waves_per_column=waves, elems_per_lane=elems, trace_cap=60,
                        teams_per_cu=teams)
    ti, tu = out["trace"].cpu().numpy().astype(np.int64) >> 6, (out["trace"].cpu().numpy().astype(np.int64) & 63) - 32
    assert np.array_equal(ti, ref["trace_i"]) and np.all(np.abs(tu) == 1) and np.all(tu[:, 1:] == -tu[:, :-1])
    assert np.array_equal(Q.cpu().numpy(), ref["Q"])


@pytest.mark.parametrize("d_out,d_in,n,bits,group,T,rq", [(24, 8200, 9000, 3, 8200, 200, False), (9, 8704, 9000, 4, 128, 300, True),
                                                          (300, 1024, 1500, 2, 1024, 150, True), (5, 64, 256, 3, 64, 40, True)])
def test_greedy_cd_two_columns_per_compute_unit(cdq, oracle, d_out, d_in, n, bits, group, T, rq):
    """Algorithm 1 with two columns resident per compute unit (Hessian diagonal in LDS, 64 registers): the oracle's moves,
    in its order, and its maintained gradient -- for the widths that take this kernel by themselves and, forced, for small ones."""
    X, Wt = rand_layer(2000 + d_in + bits, d_in, d_out, n, corr=1.0)
    H32 = oracle.hessian(X).astype(np.float32)
    a, b, q0 = oracle.init_grid(Wt, bits, group)
    if rq:
        q0 = inputs.make_random_codes(d_out, d_in, bits, seed=d_in)
    ref, Q, stats, trace, G = run_cd_both(cdq, oracle, H32, Wt, a, b, q0, bits, group, T,
                                          waves_per_column=16, elems_per_lane=16, teams_per_cu=2)
    nbad = check_cd(oracle, ref, Q, stats, trace, H32, Wt, a, b, q0, bits, group)
    if nbad == 0:
        ti, tu = decode_trace(trace)
        for j in range(d_out):
            m = ref["moves"][j]
            assert np.array_equal(ti[j, :m], ref["trace_i"][j, :m])
        assert np.array_equal(G, ref["G"])
    with pytest.raises(RuntimeError):                # the option exists for one launch shape only
        cdq.greedy_cd(dev(H32), dev(Wt), dev(a), dev(b), dev(q0.copy()), bits, group, 1, waves_per_column=8, elems_per_lane=32,
                      teams_per_cu=2)


def test_greedy_cd_alternating_for_a_long_budget(cdq, oracle):
    """A budget of 100 001 iterations: the kernel that jumps is done in microseconds, the oracle takes every step."""
    H32, Wt, ties = layer_with_exact_ties(seed=1, d_in=128, d_out=2, n=1000)
    d_out, d_in = Wt.shape
    a, b, q0 = oracle.init_grid(Wt, 3, d_in)
    T = 100001
    ref = oracle.greedy_cd(H32, Wt, a, b, q0, 3, d_in, T)
    assert np.all(ref["moves"] == T)
    Hd, Wd, ad, bd = dev(H32), dev(Wt), dev(a), dev(b)
    cdq.greedy_cd(Hd, Wd, ad, bd, dev(q0.copy()), 3, d_in, 1, waves_per_column=16, elems_per_lane=16)      # first use of this kernel
    Q = dev(q0.copy())
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    out = cdq.greedy_cd(Hd, Wd, ad, bd, Q, 3, d_in, T, waves_per_column=16, elems_per_lane=16, want_G=True)
    torch.cuda.synchronize()
    assert time.perf_counter() - t0 < 0.05, "the kernel for 16 wavefronts should not have taken every step (that takes 0.15 s)"
    assert np.array_equal(out["stats"].cpu().numpy()[:, 0], ref["moves"])
    assert np.array_equal(Q.cpu().numpy(), ref["Q"]) and np.array_equal(out["G"].cpu().numpy(), ref["G"])


# ----------------------------------------------------------------------------- OWC

@pytest.mark.parametrize("d_out,d_in,n,bits,n_gamma", [(48, 256, 600, 3, 50), (20, 1000, 1500, 4, 50), (7, 64, 200, 2, 10), (130, 128, 400, 3, 50),
                                                       # shapes that go through the fp16 look at all grid points first (d_in % 128 == 0, >= 256)
                                                       (300, 384, 900, 3, 50), (70, 1024, 1500, 2, 50), (129, 512, 800, 4, 20), (33, 256, 500, 3, 4)])
def test_init_owc(cdq, oracle, d_out, d_in, n, bits, n_gamma):
    """Eq. (2) grid search: min-max and the scale of the chosen gamma bit-exact, the chosen gamma
    equal to the oracle's exhaustive fp64 search except where two grid points have (nearly) the same loss."""
    X, Wt = rand_layer(7 + d_in, d_in, d_out, n, corr=0.5)
    rng = np.random.default_rng(d_in)
    if d_out > 60:                                   # heavy-tailed weights and channel scales: the hard case for a low-precision look
        Wt *= np.exp(0.7 * rng.standard_normal(Wt.shape)).astype(np.float32)
        X *= np.exp(0.5 * rng.standard_normal(d_in)).astype(np.float32)
    Wt[:, rng.integers(0, d_in, 3)] *= 5.0           # outlier weights make clipping pay off
    Wt[0, :] = 0.125                                 # a constant column
    H32 = oracle.hessian(X).astype(np.float32)
    a, b, q, gam, all_loss = oracle.init_owc(H32, Wt, bits, d_in, n_gamma)
    s, z, Q, g, per = cdq.init_owc(dev(H32), dev(Wt), bits, d_in, n_gamma)
    s, z, Q, g, per = (t.cpu().numpy() for t in (s, z, Q, g, per))
    # without the per-column losses the library evaluates fewer grid points in fp64; the choice must not change
    s2, z2, Q2, g2, none = cdq.init_owc(dev(H32), dev(Wt), bits, d_in, n_gamma, want_loss=False)
    assert none is None
    assert np.array_equal(g2.cpu().numpy(), g) and np.array_equal(s2.cpu().numpy(), s) and np.array_equal(Q2.cpu().numpy(), Q)
    assert np.array_equal(z, b)
    same = g == gam
    # a different gamma is acceptable only when the two grid points tie within fp32 residual rounding
    gammas = oracle.owc_gammas(n_gamma)
    for j in np.where(~same)[0]:
        k_gpu = int(np.argmin(np.abs(gammas - g[j])))
        k_ref = int(np.argmin(np.abs(gammas - gam[j])))
        assert abs(all_loss[k_gpu, j] - all_loss[k_ref, j]) <= 1e-6 * abs(all_loss[k_ref, j]) + 1e-30, (j, g[j], gam[j])
    assert same.mean() >= 0.98
    assert np.array_equal(s[same], a[same])
    assert np.array_equal(Q[same], q[same])
    ref_loss = oracle.loss(H32, Wt, q, a, b, d_in)
    np.testing.assert_allclose(per[same], ref_loss[same], rtol=1e-6, atol=1e-30)
    assert (gam < 1).any(), "the case should exercise clipping"


@pytest.mark.parametrize("kind", ["tiny_margin", "collinear_channels"])
def test_init_owc_columns_that_fail_the_check_are_searched_exhaustively(cdq, oracle, kind):
    """The fp16 look at the grid is checked column by column against the fp64 loss of the chosen grid point; a column that
    fails is searched exhaustively.  Forced two ways: a margin so small that rounding alone fails the check, and a layer
    whose input channels are nearly collinear, where fp16 cannot hold 1 - correlation and the estimate is off by percents.
    Either way the result must be the oracle's exhaustive fp64 search, and the failures must be counted."""
    d_out, d_in, n, bits, n_gamma = 96, 384, 900, 3, 50
    rng = np.random.default_rng(21)
    if kind == "collinear_channels":
        z = rng.standard_normal((n, 1)).astype(np.float32)
        X = (z + 0.05 * rng.standard_normal((n, d_in))).astype(np.float32)          # every channel is the same signal + 5 % noise
        margin = 0.0
    else:
        X, _ = rand_layer(5, d_in, d_out, n, corr=0.5)
        margin = 1e-7
    Wt = (rng.standard_normal((d_out, d_in)) / np.sqrt(d_in)).astype(np.float32)
    Wt[:, rng.integers(0, d_in, 3)] *= 5.0
    H32 = oracle.hessian(X).astype(np.float32)
    a, b, q, gam, all_loss = oracle.init_owc(H32, Wt, bits, d_in, n_gamma)
    for want_loss in (True, False):
        s, z_, Q, g, per, cnt = cdq.init_owc(dev(H32), dev(Wt), bits, d_in, n_gamma, want_loss=want_loss, screen_margin=margin,
                                            want_researched=True)
        g = g.cpu().numpy()
        n_failed = int(cnt.item())
        assert n_failed >= d_out // 3, f"only {n_failed} of {d_out} columns failed the check: the case does not exercise it"
        same = g == gam
        gammas = oracle.owc_gammas(n_gamma)
        for j in np.where(~same)[0]:                 # only exact ties of two grid points may differ
            k_gpu = int(np.argmin(np.abs(gammas - g[j])))
            k_ref = int(np.argmin(np.abs(gammas - gam[j])))
            assert abs(all_loss[k_gpu, j] - all_loss[k_ref, j]) <= 1e-6 * abs(all_loss[k_ref, j]) + 1e-30, (j, g[j], gam[j])
        assert same.mean() >= 0.97
        assert np.array_equal(s.cpu().numpy()[same], a[same]) and np.array_equal(Q.cpu().numpy()[same], q[same])
        if want_loss:
            # with collinear channels e^T H e cancels to a small fraction of |e|^2 |H|: the two sides' roundings of e show
            np.testing.assert_allclose(per.cpu().numpy()[same], all_loss.min(axis=0)[same], rtol=1e-6 if kind == "tiny_margin" else 1e-4, atol=1e-30)
    # on an ordinary layer with the default margin nothing fails
    X, _ = rand_layer(6, d_in, d_out, n, corr=0.5)
    cnt = cdq.init_owc(dev(oracle.hessian(X).astype(np.float32)), dev(Wt), bits, d_in, n_gamma, want_researched=True)[5]
    assert int(cnt.item()) == 0


@pytest.mark.parametrize("d_out,d_in,n,bits,n_gamma,margin", [(300, 384, 900, 3, 50, 0.0),      # screened: a few columns end elsewhere
                                                              (96, 384, 900, 3, 50, 1e-7),      # every column searched exhaustively
                                                              (129, 512, 800, 4, 20, 0.0), (33, 256, 500, 2, 4, 0.0),
                                                              (48, 200, 600, 3, 50, 0.0),       # no screen for this d_in
                                                              (5, 1024, 1500, 3, 50, 0.0)])
def test_init_owc_start_gradient(cdq, oracle, d_out, d_in, n, bits, n_gamma, margin):
    """The start gradient that the grid search leaves as a by-product (gradient init of Algorithm 1 for the grid of Eq. (2)
    it returns) is, bit for bit, what cdq_gradient computes for that grid; asking for it does not change the search; and
    Algorithm 1 started from it makes the moves it makes when it computes the gradient itself -- and the oracle's."""
    X, Wt = rand_layer(31 + d_in, d_in, d_out, n, corr=0.5)
    rng = np.random.default_rng(d_in + 1)
    Wt *= np.exp(0.7 * rng.standard_normal(Wt.shape)).astype(np.float32)
    Wt[:, rng.integers(0, d_in, 3)] *= 5.0
    Wt[0, :] = 0.125
    H32 = oracle.hessian(X).astype(np.float32)
    Hd, Wd = dev(H32), dev(Wt)
    s0, z0, Q0, g0, per0 = cdq.init_owc(Hd, Wd, bits, d_in, n_gamma, screen_margin=margin)
    G = torch.full((d_out, d_in), float("nan"), dtype=torch.float32, device="cuda")
    s, z, Q, g, per = cdq.init_owc(Hd, Wd, bits, d_in, n_gamma, screen_margin=margin, G_out=G)
    for u, v in ((s0, s), (z0, z), (Q0, Q), (g0, g)):
        assert torch.equal(u, v)
    np.testing.assert_allclose(per.cpu().numpy(), per0.cpu().numpy(), rtol=1e-12, atol=1e-300)     # same sums, another order
    G_ref = cdq.gradient(Hd, Wd, s, z, Q, d_in)
    assert torch.equal(G.view(torch.int32), G_ref.view(torch.int32)), "the by-product is not the gradient of the returned grid"
    # Algorithm 1 from the supplied gradient
    T = 64
    Qa, Qb = Q.clone(), Q.clone()
    out_a = cdq.greedy_cd(Hd, Wd, s, z, Qa, bits, d_in, T, want_G=True)
    out_b = cdq.greedy_cd(Hd, Wd, s, z, Qb, bits, d_in, T, want_G=True, G0=G)
    assert torch.equal(Qa, Qb) and torch.equal(out_a["stats"], out_b["stats"]) and torch.equal(out_a["G"], out_b["G"])
    ref = oracle.greedy_cd(H32, Wt, s.cpu().numpy(), z.cpu().numpy(), Q.cpu().numpy(), bits, d_in, T)
    assert np.array_equal(Qb.cpu().numpy(), ref["Q"]) and np.array_equal(out_b["stats"].cpu().numpy()[:, 0], ref["moves"])


def test_init_owc_weights_at_an_odd_address(cdq, oracle):
    """Eq. (2) grid search with Wt 4 bytes off a 16-byte boundary (the library's scalar-load kernels) chooses, for every
    column, what it chooses for the aligned copy, and that is the oracle's choice."""
    d_out, d_in, n, bits, n_gamma = 150, 384, 900, 3, 50
    X, Wt = rand_layer(77, d_in, d_out, n, corr=0.5)
    rng = np.random.default_rng(77)
    Wt *= np.exp(0.7 * rng.standard_normal(Wt.shape)).astype(np.float32)
    H32 = oracle.hessian(X).astype(np.float32)
    a, b, q, gam, all_loss = oracle.init_owc(H32, Wt, bits, d_in, n_gamma)
    Hd = dev(H32)
    buf = torch.zeros(d_out * d_in + 4, dtype=torch.float32, device="cuda")
    odd = buf[1:1 + d_out * d_in].view(d_out, d_in)
    odd.copy_(dev(Wt))
    assert odd.data_ptr() % 16 == 4 and odd.is_contiguous()
    ref = [t.cpu().numpy() for t in cdq.init_owc(Hd, dev(Wt), bits, d_in, n_gamma)]
    got = [t.cpu().numpy() for t in cdq.init_owc(Hd, odd, bits, d_in, n_gamma)]
    for r, g in zip(ref[:4], got[:4]):
        assert np.array_equal(r, g)
    np.testing.assert_allclose(got[4], ref[4], rtol=1e-9)
    same = got[3] == gam
    assert same.mean() >= 0.98
    assert np.array_equal(got[0][same], a[same]) and np.array_equal(got[1], b) and np.array_equal(got[2][same], q[same])


# ----------------------------------------------------------------------------- OWC-CD (Algorithm 3)

def owc_cd_score(oracle, H64, wj, bits, group, n_gamma, cur, i, k):
    """fp64 loss change of moving group i of one column from grid index cur[i] to k, through the oracle's Eq. (2)."""
    d_in = len(wj)
    tab = {}
    for kk in set(cur) | {k}:
        a, b, q = oracle.init_grid(wj[None, :], bits, group, float(oracle.owc_gammas(n_gamma)[kk - 1]))
        tab[kk] = oracle.residual(wj[None, :], q, a, b, group)[0].astype(np.float64)
    e = np.concatenate([tab[cur[g]][g * group:(g + 1) * group] for g in range(d_in // group)])
    sl = slice(i * group, (i + 1) * group)
    d = tab[k][sl] - e[sl]
    return float(d @ H64[sl, sl] @ d + 2.0 * (H64[sl] @ e) @ d)


@pytest.mark.parametrize("d_out,d_in,n,bits,group,n_gamma,T", [
    (40, 256, 600, 3, 32, 50, None), (9, 512, 900, 2, 128, 50, None), (17, 96, 300, 4, 8, 20, 30), (6, 128, 300, 3, 128, 50, 3),
    (5, 192, 400, 2, 64, 50, 0), (12, 1024, 1500, 3, 256, 50, None), (7, 1536, 2000, 2, 512, 12, None), (5, 120, 300, 3, 12, 50, None),
    (6, 132, 300, 3, 6, 30, None)])
@pytest.mark.parametrize("variant", [0, 1])
def test_init_owc_cd(cdq, oracle, d_out, d_in, n, bits, group, n_gamma, T, variant):
    """Algorithm 3: the sequence of (group, grid index) moves, the final strengths, grid and codes equal the
    oracle's; a column may differ only from a move on where the two candidates tie to fp64 rounding."""
    X, Wt = rand_layer(11 + d_in, d_in, d_out, n, corr=0.5)
    rng = np.random.default_rng(d_in + 1)
    Wt[:, rng.integers(0, d_in, 6)] *= 4.0
    Wt[0, :group] = 0.125                            # a constant group
    H32 = oracle.hessian(X).astype(np.float32)
    cap = (d_in // group if T is None else T) + 1
    ref = oracle.owc_cd(H32, Wt, bits, group, n_gamma, T, trace_cap=cap)
    out = {k: v.cpu().numpy() for k, v in cdq.init_owc_cd(dev(H32), dev(Wt), bits, group, n_gamma, T, trace_cap=cap, variant=variant).items()}
    assert np.array_equal(out["zero"], ref["zero"])
    H64 = H32.astype(np.float64)
    n_same = 0
    for j in range(d_out):
        gpu_moves = [(int(x) // 4096, int(x) % 4096) for x in out["trace"][j] if x >= 0]
        ref_moves = [(int(i), int(r)) for i, r in zip(ref["trace_i"][j], ref["trace_r"][j]) if i >= 0]
        if gpu_moves == ref_moves:
            n_same += 1
            assert out["moves"][j] == ref["moves"][j]
            assert np.array_equal(out["gamma_idx"][j], ref["gamma_idx"][j])
            assert np.array_equal(out["scale"][j], ref["scale"][j])
            assert np.array_equal(out["Q"][j], ref["Q"][j])
            continue
        m = next(t for t in range(max(len(gpu_moves), len(ref_moves)))
                 if t >= len(gpu_moves) or t >= len(ref_moves) or gpu_moves[t] != ref_moves[t])
        cur = [n_gamma] * (d_in // group)
        for i, k in ref_moves[:m]:
            cur[i] = k
        sg = owc_cd_score(oracle, H64, Wt[j], bits, group, n_gamma, cur, *gpu_moves[m]) if m < len(gpu_moves) else 0.0
        sr = owc_cd_score(oracle, H64, Wt[j], bits, group, n_gamma, cur, *ref_moves[m]) if m < len(ref_moves) else 0.0
        assert abs(sg - sr) <= 1e-11 * max(abs(sr), abs(sg)) + 1e-300, (j, m, gpu_moves[m:m + 1], ref_moves[m:m + 1], sg, sr)
    assert n_same >= 0.95 * d_out, n_same
    if T is None:
        assert (ref["gamma_idx"] < n_gamma).any(), "the case should exercise clipping"
    # the result is a valid Eq. (2) grid whose loss is not above MinMax's
    a0, b0, q0 = oracle.init_grid(Wt, bits, group)
    l0 = oracle.loss(H32, Wt, q0, a0, b0, group)
    l1 = oracle.loss(H32, Wt, out["Q"], out["scale"], out["zero"], group)
    assert (l1 <= l0 * (1 + 1e-9) + 1e-30).all()


def test_init_owc_cd_rejects_oversized_state(cdq):
    H = torch.zeros((16384, 16384), dtype=torch.float32, device="cuda")
    Wt = torch.zeros((1, 16384), dtype=torch.float32, device="cuda")
    with pytest.raises(RuntimeError, match="outside"):
        cdq.init_owc_cd(H, Wt, 2, 128)


# ----------------------------------------------------------------------------- BCD (Algorithm 2 / 5), k = 2

BCD_KERNELS = {"auto": {}, "single": {"single_column": True}, "wide": {"wide": True}}   # flags of cdq_bcd: the same results


def bcd_moves_from_gpu(trace_j):
    return [(int(t), int(b), int(r), np.int32(s).view(np.float32)) for t, b, r, s in trace_j if t >= 0]


@pytest.mark.parametrize("d_out,d_in,n,bits,group,T,start", [
    (24, 128, 400, 2, 128, 160, "random"), (16, 256, 700, 3, 64, 200, "random"), (10, 64, 300, 4, 16, 100, "random"),
    (12, 512, 1200, 3, 512, 300, "cd"), (9, 136, 400, 2, 8, 80, "random"), (6, 2048, 4096, 2, 128, 64, "rtn"),
    (5, 4096, 6000, 3, 4096, 24, "rtn"), (6, 3072, 4000, 3, 128, 16, "rtn"),
    # d_in not a multiple of 4: the wide-layer kernel whatever the flags
    (7, 130, 400, 3, 26, 60, "random"), (5, 1002, 1500, 4, 1002, 40, "rtn"), (3, 6, 40, 2, 6, 10, "random"), (4, 2050, 2600, 2, 410, 30, "cd"),
    # ... with 6 and with 3 columns per workgroup (what it picks for this many columns), last workgroup not full
    (1501, 130, 400, 3, 130, 24, "rtn"), (701, 66, 300, 2, 22, 20, "random"),
    # ... and with 10 and 16 columns per workgroup (rows of 16 margins)
    (2400, 66, 300, 3, 66, 20, "random"), (4000, 130, 400, 2, 26, 12, "rtn")])
@pytest.mark.parametrize("score_all,kernel", [(False, "auto"), (True, "auto"), (False, "single"), (True, "single"), (False, "wide"),
                                              (True, "wide")])
def test_bcd_vs_oracle(cdq, oracle, d_out, d_in, n, bits, group, T, start, score_all, kernel):
    """Same partitions on both sides: the trajectories (iteration, block, levels, score bits), the final codes, the
    move counts and the maintained gradient are equal bit for bit, for the kernel that gives a workgroup several
    columns, the one-column kernel and the wide-layer kernel, with and without the test that skips pairs."""
    X, Wt = rand_layer(31 + d_in + bits, d_in, d_out, n, corr=0.7)
    H32 = oracle.hessian(X).astype(np.float32)
    a, b, q_rtn = oracle.init_grid(Wt, bits, group)
    if start == "random":
        q0 = inputs.make_random_codes(d_out, d_in, bits, seed=d_in)
    elif start == "cd":                                   # the paper initialises BCD with CD
        q0 = oracle.greedy_cd(H32, Wt, a, b, q_rtn, bits, group, d_in)["Q"]
    else:
        q0 = q_rtn
    parts = inputs.make_partitions(T, d_in, seed=d_in + 1)
    ref = oracle.bcd(H32, Wt, a, b, q0, parts, bits, group, k=2, trace_cap=T)
    Q = dev(q0)
    out = cdq.bcd(dev(H32), dev(Wt), dev(a), dev(b), Q, bits, group, dev(parts), trace_cap=T, want_G=True, score_all=score_all,
                  **BCD_KERNELS[kernel])
    moves = out["moves"].cpu().numpy()
    trace = out["trace"].cpu().numpy()
    assert ref["moves"].sum() > 0
    assert np.array_equal(moves, ref["moves"])
    assert np.array_equal(Q.cpu().numpy(), ref["Q"])
    for j in range(d_out):
        got = bcd_moves_from_gpu(trace[j])
        want = [(int(t), int(bk), int(r), s) for t, bk, r, s in
                zip(ref["trace_t"][j], ref["trace_b"][j], ref["trace_r"][j], ref["trace_s"][j]) if t >= 0]
        assert [g[:3] for g in got] == [w[:3] for w in want], j
        assert all(np.float32(g[3]).tobytes() == np.float32(w[3]).tobytes() for g, w in zip(got, want)), j
    assert np.array_equal(out["G"].cpu().numpy(), ref["G"])


@pytest.mark.parametrize("T", [1, 2, 3, 5, 7])
def test_bcd_few_iterations(cdq, oracle, T):
    """Fewer iterations than the kernel's ring of partition rows has stages (its start-up and drain paths)."""
    X, Wt = rand_layer(77, 256, 11, 600, corr=0.5)
    H32 = oracle.hessian(X).astype(np.float32)
    a, b, _ = oracle.init_grid(Wt, 3, 256)
    q0 = inputs.make_random_codes(11, 256, 3, seed=T)
    parts = inputs.make_partitions(T, 256, seed=T)
    ref = oracle.bcd(H32, Wt, a, b, q0, parts, 3, 256, k=2)
    for kernel, kw in BCD_KERNELS.items():
        Q = dev(q0)
        out = cdq.bcd(dev(H32), dev(Wt), dev(a), dev(b), Q, 3, 256, dev(parts), **kw)
        assert np.array_equal(out["moves"].cpu().numpy(), ref["moves"]), kernel
        assert np.array_equal(Q.cpu().numpy(), ref["Q"]), kernel


@pytest.mark.parametrize("d_out,d_in,n,bits,T", [(4, 1360, 2313, 4, 45), (9, 336, 700, 4, 60), (5, 512, 900, 3, 50)])
def test_bcd_strongly_correlated_pairs(cdq, oracle, d_out, d_in, n, bits, T):
    """Channels of very different scale plus a common component give pairs with |H_ik| close to sqrt(H_ii H_kk); from the
    RTN start such pairs have improving moves while both coordinates are far from a single-coordinate move, the corner
    of the skip test where the product of the two 16-bit margins exceeds 2^31 (found by a randomised sweep)."""
    r = np.random.default_rng(d_in)
    X = r.standard_normal((n, d_in)).astype(np.float32) * np.exp(0.5 * r.standard_normal(d_in)).astype(np.float32)
    X += r.standard_normal((n, 1)).astype(np.float32)
    Wt = (r.standard_normal((d_out, d_in)) / np.sqrt(d_in)).astype(np.float32)
    H32 = oracle.hessian(X).astype(np.float32)
    a, b, q0 = oracle.init_grid(Wt, bits, d_in)
    parts = inputs.make_partitions(T, d_in, seed=d_in)
    ref = oracle.bcd(H32, Wt, a, b, q0, parts, bits, d_in, k=2)
    for kernel, kw in BCD_KERNELS.items():
        Q = dev(q0.copy())
        out = cdq.bcd(dev(H32), dev(Wt), dev(a), dev(b), Q, bits, d_in, dev(parts), want_G=True, **kw)
        assert np.array_equal(out["moves"].cpu().numpy(), ref["moves"]), kernel
        assert np.array_equal(Q.cpu().numpy(), ref["Q"]), kernel
        assert np.array_equal(out["G"].cpu().numpy(), ref["G"]), kernel


@pytest.mark.parametrize("d_out,d_in,n,bits,T", [(24, 512, 900, 3, 160), (10, 2048, 2600, 3, 48), (6, 1002, 1500, 3, 90), (7, 640, 900, 4, 60)])
def test_bcd_on_a_clipping_grid(cdq, oracle, d_out, d_in, n, bits, T):
    """A grid that covers half of each column's range (what a clipping initialisation gives) leaves many codes at an end
    of the grid with gradients that point past it.  The kernels' pair test counts such coordinates as unable to move on
    their own; trajectories from greedy CD's result on that grid must stay those of the oracle, which has no such test."""
    X, Wt = rand_layer(900 + d_in, d_in, d_out, n, corr=0.6)
    H32 = oracle.hessian(X).astype(np.float32)
    a, b, _ = oracle.init_grid(Wt, bits, d_in)
    top = (1 << bits) - 1
    a2 = (np.float32(0.5) * a).astype(np.float32)
    b2 = (b + np.float32(0.25 * top) * a).astype(np.float32)
    q0 = np.clip(np.rint((Wt - b2) / a2), 0, top).astype(np.uint8)
    assert ((q0 == 0) | (q0 == top)).mean() > 0.12
    q_cd = oracle.greedy_cd(H32, Wt, a2, b2, q0, bits, d_in, d_in)["Q"]
    parts = inputs.make_partitions(T, d_in, seed=d_in + 5)
    ref = oracle.bcd(H32, Wt, a2, b2, q_cd, parts, bits, d_in, k=2)
    assert ref["moves"].sum() > 0
    for kernel, kw in BCD_KERNELS.items():
        Q = dev(q_cd.copy())
        out = cdq.bcd(dev(H32), dev(Wt), dev(a2), dev(b2), Q, bits, d_in, dev(parts), want_G=True, **kw)
        assert np.array_equal(out["moves"].cpu().numpy(), ref["moves"]), kernel
        assert np.array_equal(Q.cpu().numpy(), ref["Q"]), kernel
        assert np.array_equal(out["G"].cpu().numpy(), ref["G"]), kernel


def test_bcd_rejects_bad_partitions_and_block_sizes(cdq, oracle):
    X, Wt = rand_layer(5, 64, 4, 200)
    H32 = oracle.hessian(X).astype(np.float32)
    a, b, q = oracle.init_grid(Wt, 3, 64)
    parts = inputs.make_partitions(8, 64, seed=1)
    bad = parts.copy()
    bad[3, 5] = bad[3, 6]                                  # a repeated entry: row 3 is no permutation
    Q = dev(q)
    out = cdq.bcd(dev(H32), dev(Wt), dev(a), dev(b), Q, 3, 64, dev(bad))
    assert (out["moves"].cpu().numpy() == -1).all() and np.array_equal(Q.cpu().numpy(), q)
    bad = parts.copy()
    bad[0, 0] = 64                                         # out of range
    out = cdq.bcd(dev(H32), dev(Wt), dev(a), dev(b), Q, 3, 64, dev(bad))
    assert (out["moves"].cpu().numpy() == -1).all() and np.array_equal(Q.cpu().numpy(), q)
    with pytest.raises(RuntimeError, match="outside"):
        cdq.bcd(dev(H32), dev(Wt), dev(a), dev(b), Q, 3, 64, dev(parts), k=4)
    # T = 0: nothing moves
    out = cdq.bcd(dev(H32), dev(Wt), dev(a), dev(b), Q, 3, 64, dev(parts[:0]))
    assert (out["moves"].cpu().numpy() == 0).all() and np.array_equal(Q.cpu().numpy(), q)


# ----------------------------------------------------------------------------- gradient, loss

@pytest.mark.parametrize("d_out,d_in,n,bits,group", [(64, 128, 512, 4, 128), (37, 200, 600, 3, 40), (130, 264, 800, 2, 8), (3, 7, 40, 3, 7),
                                                     (70, 1100, 1500, 3, 1100), (260, 640, 900, 4, 128)])
def test_gradient_and_loss(cdq, oracle, d_out, d_in, n, bits, group):
    X, Wt = rand_layer(d_in, d_in, d_out, n)
    H32 = oracle.hessian(X).astype(np.float32)
    a, b, q = oracle.init_grid(Wt, bits, group)
    q = np.random.default_rng(0).integers(0, 1 << bits, q.shape).astype(np.uint8)
    E = oracle.residual(Wt, q, a, b, group)
    G_ref = oracle.gradient(H32, E)
    Hd, Wd, ad, bd, qd = dev(H32), dev(Wt), dev(a), dev(b), dev(q)
    G = cdq.gradient(Hd, Wd, ad, bd, qd, group).cpu().numpy()
    diff = G != G_ref
    assert diff.mean() <= 1e-6, f"{diff.sum()} of {diff.size} gradient entries differ"
    if diff.any():
        assert np.all(np.abs(G[diff] - G_ref[diff]) <= np.spacing(np.abs(G_ref[diff])))
    per, tot = cdq.loss(Hd, Wd, ad, bd, qd, group)
    ref = oracle.loss(H32, Wt, q, a, b, group)
    # the kernel forms e in fp32 (the residual the CD arithmetic sees), the oracle in fp64
    np.testing.assert_allclose(per.cpu().numpy(), ref, rtol=1e-6)
    np.testing.assert_allclose(tot.cpu().numpy()[0], ref.sum(), rtol=1e-6)
    # with the same fp32 residual the two agree to fp64 accuracy
    E64 = E.astype(np.float64)
    ref32 = np.einsum("ji,ji->j", E64 @ H32.astype(np.float64), E64)
    np.testing.assert_allclose(per.cpu().numpy(), ref32, rtol=1e-12)


# ----------------------------------------------------------------------------- greedy CD

def decode_trace(tr):
    tr = tr.astype(np.int64)
    return tr >> 6, (tr & 63) - 32       # entries of -1 (unused slots) decode to coordinate -1


def run_cd_both(cdq, oracle, H32, Wt, a, b, q0, bits, group, T, **kw):
    ref = oracle.greedy_cd(H32, Wt, a, b, q0, bits, group, T, trace_cap=max(T, 1))
    Qd = dev(q0.copy())
    cap = max(T, 1)
    out = cdq.greedy_cd(dev(H32), dev(Wt), dev(a), dev(b), Qd, bits, group, T, trace_cap=cap, want_G=True, **kw)
    torch.cuda.synchronize()
    return ref, Qd.cpu().numpy(), out["stats"].cpu().numpy(), out["trace"].cpu().numpy(), out["G"].cpu().numpy()


def assert_divergence_is_tie(oracle, ref, trace_j, j, H32, Wt, a, b, q0, bits, group):
    """Column j ended with different codes: its first different move must be a score tie
    (the two candidates' canonical fp32 scores within 4 ulp)."""
    ti, tu = decode_trace(trace_j)
    m_ref = int(ref["moves"][j])
    k = 0
    while k < m_ref and ti[k] == ref["trace_i"][j, k]:
        # same coordinate: the level must match too (level = previous code + change)
        k += 1
    # state after the k common moves, from the oracle
    part = oracle.greedy_cd(H32, Wt[j:j + 1], a[j:j + 1], b[j:j + 1], q0[j:j + 1], bits, group, k)
    g = part["G"][0].astype(np.float64)
    qk = part["Q"][0].astype(np.int64)

    def score(i, r):
        delta = np.float32(a[j, i // group]) * np.float32(r - qk[i])
        inner = np.float32(float(delta) * float(H32[i, i]) + 2.0 * g[i])
        return np.float32(delta * inner)

    assert k < m_ref or ti[k] >= 0, "columns differ but traces do not"
    cands = []
    if k < m_ref:
        cands.append(score(int(ref["trace_i"][j, k]), int(ref["trace_r"][j, k])))
    if ti[k] >= 0:
        cands.append(score(int(ti[k]), int(qk[ti[k]] + tu[k])))
    if len(cands) == 2:
        assert abs(float(cands[0]) - float(cands[1])) <= 4 * np.spacing(np.abs(cands[0])), (j, k, cands)
    else:
        # one side stopped, the other moved: the move's score must be ~0 at rounding level
        assert abs(float(cands[0])) <= 1e-6 * float(H32[0, 0] * a[j, 0] ** 2 + 1e-30), (j, k, cands)


def check_cd(oracle, ref, Q, stats, trace, H32, Wt, a, b, q0, bits, group, min_exact=0.999):
    same = (Q == ref["Q"])
    bad_cols = np.where(~same.all(axis=1))[0]
    for j in bad_cols[:16]:
        assert_divergence_is_tie(oracle, ref, trace[j], j, H32, Wt, a, b, q0, bits, group)
    frac = same.mean()
    assert frac >= min_exact, f"only {frac:.6f} of codes equal ({len(bad_cols)} columns differ)"
    good = same.all(axis=1)
    assert np.array_equal(stats[good, 0], ref["moves"][good])
    assert np.array_equal(stats[good, 2], ref["converged"][good])
    l_gpu = oracle.loss(H32, Wt, Q, a, b, group).sum()
    l_ref = oracle.loss(H32, Wt, ref["Q"], a, b, group).sum()
    assert abs(l_gpu - l_ref) <= 1e-4 * l_ref
    return len(bad_cols)


CD_CASES = [
    # d_out, d_in, n, bits, group, T, random_q0, waves, elems
    (64, 128, 512, 4, 128, 128, False, 0, 0),
    (64, 128, 512, 4, 128, 128, True, 0, 0),
    (40, 256, 700, 3, 64, 300, True, 1, 4),
    (40, 256, 700, 3, 64, 300, True, 2, 8),
    (24, 1000, 1500, 2, 200, 500, True, 4, 4),
    (24, 1000, 1500, 4, 1000, 700, True, 1, 16),
    (16, 1030, 1500, 3, 103, 400, True, 0, 0),       # d_in % 4 != 0: scalar layout
    (9, 77, 300, 3, 11, 200, True, 4, 8),            # odd everything, more lanes than coordinates
    (12, 2048, 2600, 3, 2048, 600, True, 8, 4),
    (12, 2048, 2600, 2, 128, 600, False, 16, 4),
    (6, 4096, 4500, 4, 4096, 300, True, 2, 32),
    (6, 4096, 4500, 3, 4096, 300, True, 16, 36),     # the kernel with the Hessian diagonal in LDS (d_in above 32768)
    (7, 2048, 2600, 2, 128, 500, False, 16, 36),
    (3, 1032, 1500, 4, 8, 300, True, 16, 36),
    (5, 3072, 3600, 3, 3072, 300, True, 16, 24),     # ... and its 24- and 32-per-lane forms (d_in above 16384)
    (4, 1028, 1500, 2, 4, 400, False, 16, 24), (6, 2048, 2600, 4, 512, 300, True, 16, 32), (3, 1000, 1400, 3, 1000, 300, False, 16, 32),
    (5, 64, 256, 3, 64, 0, True, 0, 0),              # T = 0: nothing changes
    (5, 64, 256, 3, 64, 3, True, 0, 0),              # tiny budget: stops after 3 moves
    (1, 8, 64, 2, 8, 50, True, 0, 0),
]


@pytest.mark.parametrize("d_out,d_in,n,bits,group,T,rq,waves,elems", CD_CASES)
def test_greedy_cd_vs_oracle(cdq, oracle, d_out, d_in, n, bits, group, T, rq, waves, elems):
    X, Wt = rand_layer(1000 + d_in + bits, d_in, d_out, n, corr=1.0)
    H32 = oracle.hessian(X).astype(np.float32)
    a, b, q0 = oracle.init_grid(Wt, bits, group)
    if rq:
        q0 = inputs.make_random_codes(d_out, d_in, bits, seed=d_in)
    ref, Q, stats, trace, G = run_cd_both(cdq, oracle, H32, Wt, a, b, q0, bits, group, T,
                                          waves_per_column=waves, elems_per_lane=elems)
    nbad = check_cd(oracle, ref, Q, stats, trace, H32, Wt, a, b, q0, bits, group)
    if T == 0:
        assert np.array_equal(Q, q0) and not stats[:, 0].any()
    assert (stats[:, 0] <= T).all()
    if nbad == 0:
        # identical trajectories: same moves in the same order, and the same maintained gradient
        ti, tu = decode_trace(trace)
        for j in range(d_out):
            m = ref["moves"][j]
            assert np.array_equal(ti[j, :m], ref["trace_i"][j, :m])
        assert np.array_equal(G, ref["G"])


def test_greedy_cd_tiny_config_end_to_end(cdq, oracle):
    """Whole path on the tiny configuration: GPU Hessian -> RTN -> CD -> loss, against the oracle
    fed the GPU's fp32 H (stage-wise parity) and against the all-oracle run (loss only)."""
    cfg = inputs.CONFIGS["tiny"]
    X, Wt = inputs.make_layer(cfg)
    Hd = cdq.hessian(x_to_dev(X, cfg.x_dtype))
    Wd = dev(Wt)
    s, z, Q = cdq.init_rtn(Wd, cfg.bits, cfg.group)
    q0 = Q.cpu().numpy().copy()
    l0 = cdq.loss(Hd, Wd, s, z, Q, cfg.group)[1].item()
    out = cdq.greedy_cd(Hd, Wd, s, z, Q, cfg.bits, cfg.group, cfg.T)
    l1 = cdq.loss(Hd, Wd, s, z, Q, cfg.group)[1].item()
    H32 = Hd.cpu().numpy()
    ref = oracle.greedy_cd(H32, Wt, s.cpu().numpy(), z.cpu().numpy(), q0, cfg.bits, cfg.group, cfg.T)
    assert (Q.cpu().numpy() == ref["Q"]).mean() >= 0.999
    assert np.array_equal(out["stats"].cpu().numpy()[:, 0], ref["moves"])
    assert l1 <= l0
    H64 = oracle.hessian(X)
    a, b, q_rtn = oracle.init_grid(Wt, cfg.bits, cfg.group)
    full = oracle.greedy_cd(H64.astype(np.float32), Wt, a, b, q_rtn, cfg.bits, cfg.group, cfg.T)
    l_full = oracle.loss(H64, Wt, full["Q"], a, b, cfg.group).sum()
    assert abs(l1 - l_full) <= 1e-4 * l_full


def test_greedy_cd_deterministic_and_resumable(cdq, oracle):
    X, Wt = rand_layer(77, 512, 48, 1200)
    H32 = oracle.hessian(X).astype(np.float32)
    a, b, _ = oracle.init_grid(Wt, 3, 128)
    q0 = inputs.make_random_codes(48, 512, 3, seed=5)
    Hd, Wd, ad, bd = dev(H32), dev(Wt), dev(a), dev(b)
    Q1, Q2, Q3 = dev(q0.copy()), dev(q0.copy()), dev(q0.copy())
    cdq.greedy_cd(Hd, Wd, ad, bd, Q1, 3, 128, 400)
    cdq.greedy_cd(Hd, Wd, ad, bd, Q2, 3, 128, 400, waves_per_column=4, elems_per_lane=8)
    assert torch.equal(Q1, Q2), "result must not depend on the launch shape"
    cdq.greedy_cd(Hd, Wd, ad, bd, Q3, 3, 128, 150)
    st = cdq.greedy_cd(Hd, Wd, ad, bd, Q3, 3, 128, 250)["stats"]
    # resuming recomputes g from the codes in fp64, so the continued run may differ from the
    # uninterrupted one only where fp32 drift of g decided a near-tie
    assert (Q3 == Q1).float().mean().item() >= 0.999


@pytest.mark.parametrize("bits,group,rq", [(2, 128, True), (3, 1024, True), (4, 1024, False), (4, 64, True)])
def test_greedy_cd_scorers_agree(cdq, oracle, bits, group, rq):
    """The nearest-level scorer (with the two-level scorer as arbiter) and the two-level scorer
    alone must produce the same moves in the same order."""
    d_out, d_in, n, T = 96, 1024, 2048, 700
    X, Wt = rand_layer(4242 + bits, d_in, d_out, n)
    H32 = oracle.hessian(X).astype(np.float32)
    a, b, q0 = oracle.init_grid(Wt, bits, group)
    if rq:
        q0 = inputs.make_random_codes(d_out, d_in, bits, seed=bits)
    Hd, Wd, ad, bd = dev(H32), dev(Wt), dev(a), dev(b)
    Qa, Qb = dev(q0.copy()), dev(q0.copy())
    oa = cdq.greedy_cd(Hd, Wd, ad, bd, Qa, bits, group, T, trace_cap=T, want_G=True)
    ob = cdq.greedy_cd(Hd, Wd, ad, bd, Qb, bits, group, T, trace_cap=T, want_G=True, exact_scorer_only=True)
    assert torch.equal(Qa, Qb)
    assert torch.equal(oa["trace"], ob["trace"])
    assert torch.equal(oa["G"], ob["G"])
    assert torch.equal(oa["stats"], ob["stats"])


def test_greedy_cd_dead_channel_and_diagonal(cdq, oracle):
    # dead input channels (H_ii = 0, a zero row of H): never selected, no NaN -- in every kernel family, with both scorers
    # (the kernels that keep the diagonal in LDS divide by the curvature without a guard and rely on the comparison with a
    # score that is not a number being false)
    X, Wt = rand_layer(5, 64, 8, 300)
    X[:, 9] = 0
    X[:, 40] = 0
    H32 = oracle.hessian(X).astype(np.float32)
    a, b, _ = oracle.init_grid(Wt, 3, 64)
    q0 = inputs.make_random_codes(8, 64, 3, seed=1)
    for waves, elems, teams in ((0, 0, 0), (1, 16, 0), (16, 16, 1), (16, 16, 2), (16, 24, 0), (16, 32, 0), (16, 36, 0)):
        for exact in (False, True):
            ref, Q, stats, trace, G = run_cd_both(cdq, oracle, H32, Wt, a, b, q0, 3, 64, 200, waves_per_column=waves, elems_per_lane=elems,
                                                  teams_per_cu=teams, exact_scorer_only=exact)
            assert np.array_equal(Q, ref["Q"]) and np.array_equal(Q[:, [9, 40]], q0[:, [9, 40]]) and np.isfinite(G).all(), (waves, elems, teams, exact)
            assert np.array_equal(stats[:, 0], ref["moves"]) and np.array_equal(G, ref["G"])
    # diagonal H: CD from arbitrary codes lands exactly on round-to-nearest
    Hdiag = np.diag(np.random.default_rng(2).uniform(0.5, 4, 64)).astype(np.float32)
    a, b, q_rtn = oracle.init_grid(Wt, 4, 64)
    q0 = inputs.make_random_codes(8, 64, 4, seed=2)
    Qd = dev(q0.copy())
    cdq.greedy_cd(dev(Hdiag), dev(Wt), dev(a), dev(b), Qd, 4, 64, 128)
    assert np.array_equal(Qd.cpu().numpy(), q_rtn)


@pytest.mark.parametrize("d_out,d_in,n,bits,group", [(33, 200, 500, 3, 40), (16, 1024, 1500, 4, 1024), (5, 77, 300, 2, 7)])
def test_single_steps_match_oracle(cdq, oracle, d_out, d_in, n, bits, group):
    """The arg-min step and the update step of one iteration, each against the oracle."""
    X, Wt = rand_layer(900 + d_in, d_in, d_out, n)
    H32 = oracle.hessian(X).astype(np.float32)
    a, b, _ = oracle.init_grid(Wt, bits, group)
    q0 = inputs.make_random_codes(d_out, d_in, bits, seed=d_out)
    E = oracle.residual(Wt, q0, a, b, group)
    G0 = oracle.gradient(H32, E)
    ri, rr, rs = oracle.argmin_step(np.diag(H32).copy(), a, q0, G0, bits, group)
    Hd, ad, Qd, Gd = dev(H32), dev(a), dev(q0.copy()), dev(G0.copy())
    bi, br, bs = cdq.score_argmin(dev(np.diag(H32).copy()), ad, Qd, Gd, bits, group)
    assert np.array_equal(bi.cpu().numpy(), ri) and np.array_equal(br.cpu().numpy(), rr)
    assert np.array_equal(bs.cpu().numpy(), rs)
    moves = torch.zeros(d_out, dtype=torch.int32, device="cuda")
    cdq.gather_update(Hd, ad, Qd, Gd, group, bi, br, moves)
    one = oracle.greedy_cd(H32, Wt, a, b, q0, bits, group, 1)
    assert np.array_equal(Qd.cpu().numpy(), one["Q"])
    assert np.array_equal(Gd.cpu().numpy(), one["G"])
    assert np.array_equal(moves.cpu().numpy(), one["moves"])
    # a column with no improving move is reported as such and left untouched
    Hdiag = np.diag(np.full(d_in, 2.0)).astype(np.float32)
    a1, b1, q_rtn = oracle.init_grid(Wt, bits, group)
    G1 = oracle.gradient(Hdiag, oracle.residual(Wt, q_rtn, a1, b1, group))
    bi, br, bs = cdq.score_argmin(dev(np.full(d_in, 2.0, np.float32)), dev(a1), dev(q_rtn), dev(G1), bits, group)
    assert (bi.cpu().numpy() == -1).all() and (bs.cpu().numpy() == 0).all()


def test_stepwise_loop_equals_fused(cdq, oracle):
    """2T separate launches give the same codes and move counts as the fused persistent kernel."""
    d_out, d_in, n, bits, group, T = 40, 520, 1200, 3, 104, 150
    X, Wt = rand_layer(31, d_in, d_out, n)
    H32 = oracle.hessian(X).astype(np.float32)
    a, b, _ = oracle.init_grid(Wt, bits, group)
    q0 = inputs.make_random_codes(d_out, d_in, bits, seed=3)
    Hd, Wd, ad, bd = dev(H32), dev(Wt), dev(a), dev(b)
    Qf, Qs = dev(q0.copy()), dev(q0.copy())
    st = cdq.greedy_cd(Hd, Wd, ad, bd, Qf, bits, group, T)["stats"]
    mv = cdq.greedy_cd_stepwise(Hd, Wd, ad, bd, Qs, bits, group, T)
    assert torch.equal(Qf, Qs)
    assert torch.equal(st[:, 0], mv)
    ref = oracle.greedy_cd(H32, Wt, a, b, q0, bits, group, T)
    assert np.array_equal(Qs.cpu().numpy(), ref["Q"])


def test_empty_layer(cdq):
    H = torch.zeros((8, 8), device="cuda")
    Wt = torch.zeros((0, 8), device="cuda")
    s, z, Q = cdq.init_rtn(Wt, 3, 8)
    assert Q.shape == (0, 8)
    out = cdq.greedy_cd(H, Wt, s, z, Q, 3, 8, 4)
    per, tot = cdq.loss(H, Wt, s, z, Q, 8)
    assert per.numel() == 0 and tot.item() == 0.0


# ----------------------------------------------------------------------------- streaming layer driver

@pytest.mark.parametrize("init,bits,group,with_bcd", [("rtn", 3, 256, True), ("owc", 4, 256, False), ("owc_cd", 2, 64, False)])
def test_layer_driver_streams_chunks_and_matches_oracle(cdq, oracle, init, bits, group, with_bcd):
    """quantize_layer over ragged token chunks: the accumulated, damped H matches the fp64 oracle on all tokens; with that H
    the oracle reproduces the start, the CD codes and (when asked) the BCD codes; the reported losses are the oracle's."""
    from paper_2406_17542_amd import layer
    d_in, d_out, n = 256, 40, 2000
    X = inputs.make_x("student_t4", n, d_in, seed=4, x_dtype="bf16")
    Wt = inputs.make_wt(d_out, d_in, 5)
    Wt[:, ::37] *= 3.0
    Xd = x_to_dev(X, "bf16")
    cuts = [0, 512, 1300, 1301, n]
    chunks = [Xd[a:b].contiguous() for a, b in zip(cuts[:-1], cuts[1:])]
    parts = inputs.make_partitions(48, d_in, seed=6)
    r = layer.quantize_layer(iter(chunks), dev(Wt), bits, group, T=d_in, init=init, lambda_rel=0.01,
                             bcd_parts=dev(parts) if with_bcd else None)
    assert r["n_tokens"] == n
    H = r["H"].cpu().numpy()
    ok, worst, fro = hessian_tolerance_ok(H, oracle.hessian(X, lambda_rel=0.01), n)
    assert ok and fro <= 1e-5, (worst, fro)
    if init == "rtn":
        a, b, q0 = oracle.init_grid(Wt, bits, group)
    elif init == "owc":
        a, b, q0, _, _ = oracle.init_owc(H, Wt, bits, group, 50)
    else:
        o = oracle.owc_cd(H, Wt, bits, group, 50)
        a, b, q0 = o["scale"], o["zero"], o["Q"]
    assert np.array_equal(r["scale"].cpu().numpy(), a) and np.array_equal(r["zero"].cpu().numpy(), b)
    np.testing.assert_allclose(r["loss_init"], oracle.loss(H, Wt, q0, a, b, group).sum(), rtol=1e-6)
    ref = oracle.greedy_cd(H, Wt, a, b, q0, bits, group, d_in)
    np.testing.assert_allclose(r["loss_cd"], oracle.loss(H, Wt, ref["Q"], a, b, group).sum(), rtol=1e-6)
    q_ref = ref["Q"]
    if with_bcd:
        q_ref = oracle.bcd(H, Wt, a, b, ref["Q"], parts, bits, group, k=2)["Q"]
        np.testing.assert_allclose(r["loss_bcd"], oracle.loss(H, Wt, q_ref, a, b, group).sum(), rtol=1e-6)
        assert r["loss_bcd"] <= r["loss_cd"]
    assert (r["Q"].cpu().numpy() == q_ref).mean() >= 0.999
    assert r["loss_cd"] <= r["loss_init"]
    assert set(r["seconds"]) >= {"hessian", "init", "cd", "loss"}


# ----------------------------------------------------------------------------- cyclic CD

@pytest.mark.parametrize("d_out,d_in,n,bits,group,T,start", [
    (20, 128, 400, 3, 128, 1280, "random"), (12, 520, 1200, 2, 40, 1500, "random"), (9, 64, 300, 4, 16, 64, "random"),
    (16, 2048, 4096, 3, 2048, 6144, "rtn"), (7, 300, 700, 4, 300, 100, "rtn"), (5, 1024, 2000, 2, 128, 0, "rtn")])
def test_cyclic_cd_vs_oracle(cdq, oracle, d_out, d_in, n, bits, group, T, start):
    """Fixed-order CD: moves (coordinate, level), codes, visit counts, convergence flags and the maintained gradient
    are bit-equal to the oracle's."""
    X, Wt = rand_layer(50 + d_in + bits, d_in, d_out, n, corr=0.0 if d_in == 128 else 0.6)
    H32 = oracle.hessian(X).astype(np.float32)
    a, b, q_rtn = oracle.init_grid(Wt, bits, group)
    q0 = inputs.make_random_codes(d_out, d_in, bits, seed=d_in) if start == "random" else q_rtn
    cap = max(T, 1)
    ref = oracle.cyclic_cd(H32, Wt, a, b, q0, bits, group, T, trace_cap=cap)
    Q = dev(q0)
    out = cdq.cyclic_cd(dev(H32), dev(Wt), dev(a), dev(b), Q, bits, group, T, trace_cap=cap, want_G=True)
    st = out["stats"].cpu().numpy()
    assert np.array_equal(st[:, 0], ref["moves"])
    assert np.array_equal(st[:, 1], ref["iters"])
    assert np.array_equal(st[:, 2], ref["converged"])
    assert np.array_equal(Q.cpu().numpy(), ref["Q"])
    tr = out["trace"].cpu().numpy()
    for j in range(d_out):
        m = ref["moves"][j]
        assert np.array_equal(tr[j, :m] >> 7, ref["trace_i"][j, :m])
        assert np.array_equal(tr[j, :m] & 127, ref["trace_r"][j, :m])
    assert np.array_equal(out["G"].cpu().numpy(), ref["G"])
    if d_in == 128:
        assert ref["converged"].any(), "ten epochs on the uncorrelated case should reach a coordinate-wise optimum"


# ----------------------------------------------------------------------------- randomised shapes

def scaled_layer(seed, d_in, d_out, n, corr):
    """Channels of very different scale plus a common component: strongly correlated pairs, large and small H_ii."""
    r = np.random.default_rng(seed)
    X = r.standard_normal((n, d_in)).astype(np.float32) * np.exp(0.5 * r.standard_normal(d_in)).astype(np.float32)
    if corr:
        X += (corr * r.standard_normal((n, 1))).astype(np.float32)
    Wt = (r.standard_normal((d_out, d_in)) / np.sqrt(d_in)).astype(np.float32)
    return X, Wt


@pytest.mark.parametrize("seed,big", [(1, False), (2, False), (3, True)])
def test_random_shapes_against_the_oracle(cdq, oracle, seed, big):
    """A seeded sweep over shapes nobody picked by hand (widths, group sizes, column counts, budgets, starts): greedy CD,
    block CD (both kernels, with and without the pair test), cyclic CD, loss and gradient against the oracle, exactly."""
    rng = np.random.default_rng(seed)
    for case in range(45 if big else 120):
        bits = int(rng.choice([2, 3, 4]))
        kind = str(rng.choice(["cd", "cd", "bcd", "bcd", "cyclic", "loss"]))
        d_in = int(rng.integers(2, 90)) * int(rng.choice([16, 32, 48] if big else [2, 4, 8, 16, 16]))
        divs = [g for g in range(1, d_in + 1) if d_in % g == 0]
        group = int(rng.choice(divs[len(divs) // 2:]))
        d_out = int(rng.integers(1, 40))
        n = int(rng.integers(d_in, 3 * d_in + 8))
        corr = float(rng.choice([0.0, 0.5, 1.0]))
        X, Wt = scaled_layer(1000 * seed + case, d_in, d_out, n, corr)
        H32 = oracle.hessian(X).astype(np.float32)
        a, b, q_rtn = oracle.init_grid(Wt, bits, group)
        q0 = q_rtn if rng.random() < 0.5 else inputs.make_random_codes(d_out, d_in, bits, seed=case)
        tag = f"case {case}: {kind} d_out={d_out} d_in={d_in} n={n} bits={bits} group={group} corr={corr}"
        Hd, Wd, ad, bd = dev(H32), dev(Wt), dev(a), dev(b)
        if kind == "cd":
            T = int(rng.integers(1, 2 * d_in))
            ref = oracle.greedy_cd(H32, Wt, a, b, q0, bits, group, T)
            Q = dev(q0.copy())
            out = cdq.greedy_cd(Hd, Wd, ad, bd, Q, bits, group, T)
            assert np.array_equal(Q.cpu().numpy(), ref["Q"]), tag
            assert np.array_equal(out["stats"].cpu().numpy()[:, 0], ref["moves"]), tag
        elif kind == "bcd":
            T = int(rng.integers(1, 60))
            parts = inputs.make_partitions(T, d_in, seed=case)
            ref = oracle.bcd(H32, Wt, a, b, q0, parts, bits, group, k=2)
            for kernel, kw in BCD_KERNELS.items():
                for score_all in (False, True):
                    Q = dev(q0.copy())
                    out = cdq.bcd(Hd, Wd, ad, bd, Q, bits, group, dev(parts), score_all=score_all, want_G=True, **kw)
                    assert np.array_equal(Q.cpu().numpy(), ref["Q"]), (tag, kernel, score_all)
                    assert np.array_equal(out["moves"].cpu().numpy(), ref["moves"]), (tag, kernel, score_all)
                    assert np.array_equal(out["G"].cpu().numpy(), ref["G"]), (tag, kernel, score_all)
        elif kind == "cyclic":
            T = int(rng.integers(1, 3 * d_in))
            ref = oracle.cyclic_cd(H32, Wt, a, b, q0, bits, group, T)
            Q = dev(q0.copy())
            cdq.cyclic_cd(Hd, Wd, ad, bd, Q, bits, group, T)
            assert np.array_equal(Q.cpu().numpy(), ref["Q"]), tag
        else:
            E = oracle.residual(Wt, q0, a, b, group)
            E64 = E.astype(np.float64)
            ref = np.einsum("ji,ji->j", E64 @ H32.astype(np.float64), E64)
            per = cdq.loss(Hd, Wd, ad, bd, dev(q0), group)[0].cpu().numpy()
            np.testing.assert_allclose(per, ref, rtol=1e-11, err_msg=tag)
            G = cdq.gradient(Hd, Wd, ad, bd, dev(q0), group).cpu().numpy()
            assert (G != oracle.gradient(H32, E)).mean() <= 1e-5, tag
