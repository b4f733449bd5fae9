"""Parity at the real shapes, in the launch configuration bench.py times (default launch shape,
whole layer on the GPU), checked on sampled outputs the oracle can compute one by one:
  * Hessian: the whole diagonal and 4096 random entries recomputed from X in fp64
  * greedy CD: a random sample of columns rerun by the oracle from the same fp32 H -- codes,
    move counts and convergence flags must match (>= 99.9 % of codes; in practice all)
  * loss: per-column values of the sampled columns against the oracle's fp64 loss
and on properties that hold at any size (loss never increases, every column reports convergence
or exhausts T, H symmetric).  Each test prints its steps so a long run is visibly alive.
"""
import time

import numpy as np
import pytest
import torch

from paper_2406_17542_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def cdq():
    assert torch.cuda.is_available()
    from paper_2406_17542_amd import cdq as m
    m.lib()
    return m


def say(msg):
    print(f"[{time.strftime('%H:%M:%S')}] {msg}", flush=True)


def x_to_dev(X, x_dtype):
    if x_dtype == "bf16":
        return torch.from_numpy(inputs.bf16_bits(X).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(X).cuda()


def check_hessian_samples(H, X, n_samples=4096, seed=0):
    """Diagonal and random entries of H against fp64 sums over the tokens of X."""
    n, d_in = X.shape
    rng = np.random.default_rng(seed)
    diag = np.einsum("ti,ti->i", X, X, dtype=np.float64)
    Hd = np.diag(H).astype(np.float64)
    tol = 8.0 * np.sqrt(n) * 2.0 ** -24
    assert np.all(np.abs(Hd - diag) <= tol * diag + 1e-30)
    ii = rng.integers(0, d_in, n_samples)
    kk = rng.integers(0, d_in, n_samples)
    ref = np.einsum("ts,ts->s", X[:, ii].astype(np.float64), X[:, kk].astype(np.float64))
    err = np.abs(H[ii, kk].astype(np.float64) - ref)
    assert np.all(err <= tol * np.sqrt(diag[ii] * diag[kk]) + 1e-30), float((err / (tol * np.sqrt(diag[ii] * diag[kk]))).max())
    assert np.array_equal(H[ii, kk], H[kk, ii])


def recheck_diverged_columns(cdq, oracle, Hd, H32, Wt, a, b, q0, cols_bad, bits, group, T, shape):
    """Columns whose final codes differ from the oracle's: rerun them on the GPU with a move trace, in the launch
    shape of the full run, and require the first different move to be a tie of the two candidates' scores."""
    from test_gpu_parity import assert_divergence_is_tie
    for j in cols_bad:
        sl = slice(j, j + 1)
        Qd = torch.from_numpy(q0[sl].copy()).cuda()
        out = cdq.greedy_cd(Hd, torch.from_numpy(np.ascontiguousarray(Wt[sl])).cuda(), torch.from_numpy(a[sl].copy()).cuda(),
                            torch.from_numpy(b[sl].copy()).cuda(), Qd, bits, group, T, trace_cap=T,
                            waves_per_column=shape[0], elems_per_lane=shape[1])
        ref = oracle.greedy_cd(H32, Wt[sl], a[sl], b[sl], q0[sl], bits, group, T, trace_cap=T)
        assert_divergence_is_tie(oracle, ref, out["trace"].cpu().numpy()[0], 0, H32, Wt[sl], a[sl], b[sl], q0[sl], bits, group)


def run_layer(cdq, oracle, cfg, d_out, T, sample_cols, q0_random=False, seed=0, include_busiest=0):
    say(f"{cfg.name}: generating X [{cfg.n}x{cfg.d_in}] and Wt [{d_out}x{cfg.d_in}]")
    X, Wt = inputs.make_layer(cfg, d_out=d_out)
    Xd = x_to_dev(X, cfg.x_dtype)
    say("hessian on the GPU")
    Hd = cdq.hessian(Xd)
    H32 = Hd.cpu().numpy()
    say("hessian spot checks in fp64")
    check_hessian_samples(H32, X)
    del Xd
    Wd = torch.from_numpy(Wt).cuda()
    scale, zero, Q = cdq.init_rtn(Wd, cfg.bits, cfg.group)
    a, b, q_rtn = oracle.init_grid(Wt, cfg.bits, cfg.group)
    assert np.array_equal(Q.cpu().numpy(), q_rtn), "RTN codes differ"
    assert np.array_equal(scale.cpu().numpy(), a) and np.array_equal(zero.cpu().numpy(), b)
    if q0_random:
        q0 = inputs.make_random_codes(d_out, cfg.d_in, cfg.bits, seed=cfg.seed)
        Q.copy_(torch.from_numpy(q0).cuda())
    else:
        q0 = q_rtn
    l0 = cdq.loss(Hd, Wd, scale, zero, Q, cfg.group)[0].cpu().numpy()
    say(f"greedy CD on the GPU, T={T}, default launch shape")
    out = cdq.greedy_cd(Hd, Wd, scale, zero, Q, cfg.bits, cfg.group, T)
    torch.cuda.synchronize()
    l1 = cdq.loss(Hd, Wd, scale, zero, Q, cfg.group)[0].cpu().numpy()
    stats = out["stats"].cpu().numpy()
    Qn = Q.cpu().numpy()
    # properties that hold at any size
    assert np.all(l1 <= l0 * (1 + 1e-9)), "loss increased on some column"
    assert np.all((stats[:, 2] == 1) | (stats[:, 0] == T)), "a column neither converged nor used its budget"
    assert np.all(stats[:, 0] <= T)
    changed = (Qn != q0).sum(axis=1)
    assert np.all(changed <= stats[:, 0])
    # sampled columns through the oracle
    rng = np.random.default_rng(seed + 1)
    cols = rng.choice(d_out, size=min(sample_cols, d_out), replace=False)
    if include_busiest:                 # the longest trajectories are where drift of the gradient would show
        cols = np.concatenate([cols, np.argsort(-stats[:, 0], kind="stable")[:include_busiest]])
    cols = np.unique(cols)
    say(f"oracle on {len(cols)} sampled columns for the full T={T} (most moves in the sample: {int(stats[cols, 0].max())})")
    ref = oracle.greedy_cd(H32, Wt[cols], a[cols], b[cols], q0[cols], cfg.bits, cfg.group, T)
    same = Qn[cols] == ref["Q"]
    frac = same.mean()
    say(f"codes equal on {frac:.6f} of sampled entries; moves total {int(stats[:, 0].sum())}, "
        f"mean {stats[:, 0].mean():.1f}, max {stats[:, 0].max()}, converged {int(stats[:, 2].sum())}/{d_out}")
    assert frac >= 0.999
    good = same.all(axis=1)
    assert good.mean() >= 0.98, "too many sampled columns diverged"
    if not good.all():
        say(f"columns {cols[~good].tolist()} differ: checking that each diverges at a tie")
        recheck_diverged_columns(cdq, oracle, Hd, H32, Wt, a, b, q0, cols[~good].tolist(), cfg.bits, cfg.group, T,
                                 cdq.greedy_cd_shape(d_out, cfg.d_in, cfg.group))
    assert np.array_equal(stats[cols][good, 0], ref["moves"][good])
    assert np.array_equal(stats[cols][good, 2], ref["converged"][good])
    l_ref = oracle.loss(H32, Wt[cols], ref["Q"], a[cols], b[cols], cfg.group)
    np.testing.assert_allclose(l1[cols][good], l_ref[good], rtol=1e-6)
    assert abs(l1[cols].sum() - l_ref.sum()) <= 1e-4 * l_ref.sum()
    return stats


def test_attn_proj_full_layer(cdq, oracle):
    """The benchmark workload itself: whole layer, full T, RTN start."""
    cfg = inputs.CONFIGS["attn_proj"]
    stats = run_layer(cdq, oracle, cfg, cfg.d_out, cfg.T, sample_cols=160)
    assert stats[:, 2].all(), "every column of this layer converges well before T = d_in"


def test_attn_proj_random_start(cdq, oracle):
    """Same layer from uniform random codes: every column uses its whole budget."""
    cfg = inputs.CONFIGS["attn_proj"]
    run_layer(cdq, oracle, cfg, 512, 1024, sample_cols=48, q0_random=True)


def test_mlp_up_column_subset(cdq, oracle):
    """2-bit, groups of 128, Student-t activations; 2048 of the 16384 columns, full T."""
    cfg = inputs.CONFIGS["mlp_up"]
    run_layer(cdq, oracle, cfg, 2048, cfg.T, sample_cols=160)


def test_mlp_down_column_subset(cdq, oracle):
    """d_in = 16384 (H is 1 GiB): 512 columns -- more than there are compute units, so the kernel is the one the full layer
    takes, two columns per compute unit -- for the configured T = 16384; the oracle reruns 10 random columns and the 4 with
    the most moves (several thousand each) for that full budget."""
    cfg = inputs.CONFIGS["mlp_down"]
    assert cdq.greedy_cd_shape(512, cfg.d_in, cfg.group) == cdq.greedy_cd_shape(cfg.d_out, cfg.d_in, cfg.group)
    stats = run_layer(cdq, oracle, cfg, 512, cfg.T, sample_cols=10, include_busiest=4)
    assert stats[:, 0].max() > 2000, "the sample should contain long trajectories"


def test_large_owc_init_column_subset(cdq, oracle):
    """d_in = 8192, 3-bit per-channel with the scale chosen by OWC (grid of 50), then greedy CD for the configured
    T = 8192: 256 columns on the GPU in the full layer's launch shape; 12 of them (8 random, the 4 with the most
    moves) through the oracle's exhaustive fp64 grid search and its full-T CD."""
    cfg = inputs.CONFIGS["large"]
    d_out, T = 256, cfg.T
    assert cdq.greedy_cd_shape(d_out, cfg.d_in, cfg.group) == cdq.greedy_cd_shape(cfg.d_out, cfg.d_in, cfg.group)
    say(f"{cfg.name}: generating X [{cfg.n}x{cfg.d_in}] and Wt [{d_out}x{cfg.d_in}]")
    X, Wt = inputs.make_layer(cfg, d_out=d_out)
    Xd = x_to_dev(X, cfg.x_dtype)
    Hd = cdq.hessian(Xd)
    H32 = Hd.cpu().numpy()
    say("hessian spot checks in fp64")
    check_hessian_samples(H32, X, n_samples=1024)
    del Xd, X
    Wd = torch.from_numpy(Wt).cuda()
    say("OWC grid search on the GPU")
    scale, zero, Q, gamma, per = cdq.init_owc(Hd, Wd, cfg.bits, cfg.group, 50)
    # bench.py does not ask for the per-column losses, which takes another path through the search: same choice
    # ... and has the search hand over the start gradient of Algorithm 1, which the run below then starts from
    G0 = torch.empty((d_out, cfg.d_in), dtype=torch.float32, device="cuda")
    s_b, z_b, Q_b, gamma_b, _ = cdq.init_owc(Hd, Wd, cfg.bits, cfg.group, 50, want_loss=False, G_out=G0)
    assert torch.equal(gamma_b, gamma) and torch.equal(s_b, scale) and torch.equal(Q_b, Q)
    assert torch.equal(G0, cdq.gradient(Hd, Wd, scale, zero, Q, cfg.group))
    del s_b, z_b, Q_b, gamma_b
    s_rtn, z_rtn, Q_rtn = cdq.init_rtn(Wd, cfg.bits, cfg.group)
    l_rtn = cdq.loss(Hd, Wd, s_rtn, z_rtn, Q_rtn, cfg.group)[0]
    assert torch.all(per <= l_rtn * (1 + 1e-9)), "gamma = 1 is on the grid, so OWC can not be worse than MinMax"
    q0 = Q.cpu().numpy().copy()
    say(f"greedy CD on the GPU, T={T}")
    out = cdq.greedy_cd(Hd, Wd, scale, zero, Q, cfg.bits, cfg.group, T, G0=G0)
    del G0
    l1 = cdq.loss(Hd, Wd, scale, zero, Q, cfg.group)[0].cpu().numpy()
    assert np.all(l1 <= per.cpu().numpy() * (1 + 1e-9))
    stats = out["stats"].cpu().numpy()
    assert np.all((stats[:, 2] == 1) | (stats[:, 0] == T))
    cols = np.unique(np.concatenate([np.random.default_rng(5).choice(d_out, size=8, replace=False),
                                     np.argsort(-stats[:, 0], kind="stable")[:4]]))
    say(f"oracle OWC (exhaustive fp64 search) + CD for T={T} on {len(cols)} sampled columns; most moves in the sample {int(stats[cols, 0].max())}")
    a, b, q, gam, l_all = oracle.init_owc(H32, Wt[cols], cfg.bits, cfg.group, 50)
    l_owc = l_all.min(axis=0)                     # [n_gamma][columns] -> the loss of each column's best grid point
    g_gpu = gamma.cpu().numpy()[cols]
    same = g_gpu == gam
    say(f"gamma equal on {int(same.sum())}/{len(cols)} sampled columns; gamma range {gam.min():.2f}..{gam.max():.2f}")
    # a different clipping strength is acceptable only where the two grid points' losses tie
    per_n = per.cpu().numpy()
    for c in np.where(~same)[0]:
        assert abs(per_n[cols[c]] - l_owc[c]) <= 1e-6 * l_owc[c], (int(cols[c]), float(g_gpu[c]), float(gam[c]))
    assert same.sum() >= len(cols) - 1
    np.testing.assert_allclose(per_n[cols][same], l_owc[same], rtol=1e-6)
    assert np.array_equal(scale.cpu().numpy()[cols][same, 0], a[same, 0])
    assert np.array_equal(q0[cols][same], q[same])
    cs = cols[same]
    ref = oracle.greedy_cd(H32, Wt[cs], a[same], b[same], q[same], cfg.bits, cfg.group, T)
    Qn = Q.cpu().numpy()
    eq = Qn[cs] == ref["Q"]
    say(f"CD codes equal on {eq.mean():.6f} of sampled entries; moves per sampled column {stats[cs, 0].tolist()}")
    assert eq.mean() >= 0.999
    good = eq.all(axis=1)
    if not good.all():
        say(f"columns {cs[~good].tolist()} differ: checking that each diverges at a tie")
        recheck_diverged_columns(cdq, oracle, Hd, H32, Wt, scale.cpu().numpy(), zero.cpu().numpy(), q0, cs[~good].tolist(),
                                 cfg.bits, cfg.group, T, cdq.greedy_cd_shape(d_out, cfg.d_in, cfg.group))
    assert np.array_equal(stats[cs][good, 0], ref["moves"][good])
    assert np.array_equal(stats[cs][good, 2], ref["converged"][good])
    l_ref = oracle.loss(H32, Wt[cs], ref["Q"], a[same], b[same], cfg.group)
    np.testing.assert_allclose(l1[cs][good], l_ref[good], rtol=1e-6)
    assert abs(l1[cs].sum() - l_ref.sum()) <= 1e-4 * l_ref.sum()


def test_mlp_up_owc_cd_init(cdq, oracle):
    """Algorithm 3 at the real shape: all 16384 columns of the 2-bit, group-128 layer on the GPU with T = d_in/group,
    48 sampled columns through the oracle (strengths, grid and codes equal), then greedy CD from that start."""
    cfg = inputs.CONFIGS["mlp_up"]
    say(f"{cfg.name}: generating X [{cfg.n}x{cfg.d_in}] and Wt [{cfg.d_out}x{cfg.d_in}]")
    X, Wt = inputs.make_layer(cfg)
    Hd = cdq.hessian(x_to_dev(X, cfg.x_dtype))
    H32 = Hd.cpu().numpy()
    del X
    Wd = torch.from_numpy(Wt).cuda()
    say("OWC-CD on the GPU, whole layer")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    out = cdq.init_owc_cd(Hd, Wd, cfg.bits, cfg.group, 50)
    torch.cuda.synchronize()
    say(f"  {1e3 * (time.perf_counter() - t0):.1f} ms, {int(out['moves'].sum())} strength moves")
    s_rtn, z_rtn, Q_rtn = cdq.init_rtn(Wd, cfg.bits, cfg.group)
    l_rtn = cdq.loss(Hd, Wd, s_rtn, z_rtn, Q_rtn, cfg.group)[0]
    l_owc = cdq.loss(Hd, Wd, out["scale"], out["zero"], out["Q"], cfg.group)[0]
    assert torch.all(l_owc <= l_rtn * (1 + 1e-9)), "every move lowers the loss, so the result can not be worse than MinMax"
    say(f"  layer loss MinMax {float(l_rtn.sum()):.6e} -> OWC-CD {float(l_owc.sum()):.6e}")
    assert float(l_owc.sum()) < float(l_rtn.sum())
    gi = out["gamma_idx"].cpu().numpy()
    assert gi.min() >= 1 and gi.max() <= 50
    assert np.array_equal((gi != 50).sum(axis=1) <= out["moves"].cpu().numpy(), np.ones(cfg.d_out, bool))
    cols = np.sort(np.random.default_rng(9).choice(cfg.d_out, size=48, replace=False))
    say(f"oracle OWC-CD on {len(cols)} sampled columns")
    ref = oracle.owc_cd(H32, Wt[cols], cfg.bits, cfg.group, 50)
    same = (gi[cols] == ref["gamma_idx"]).all(axis=1)
    say(f"  strengths equal on {int(same.sum())}/{len(cols)} sampled columns")
    assert same.sum() >= len(cols) - 1
    assert np.array_equal(out["scale"].cpu().numpy()[cols][same], ref["scale"][same])
    assert np.array_equal(out["zero"].cpu().numpy()[cols], ref["zero"])
    assert np.array_equal(out["Q"].cpu().numpy()[cols][same], ref["Q"][same])
    assert np.array_equal(out["moves"].cpu().numpy()[cols][same], ref["moves"][same])
    say("greedy CD from the OWC-CD start")
    Q = out["Q"].clone()
    cdq.greedy_cd(Hd, Wd, out["scale"], out["zero"], Q, cfg.bits, cfg.group, cfg.T)
    l_cd = cdq.loss(Hd, Wd, out["scale"], out["zero"], Q, cfg.group)[0]
    assert torch.all(l_cd <= l_owc * (1 + 1e-9))
    refcd = oracle.greedy_cd(H32, Wt[cols][same], ref["scale"][same], ref["zero"][same], ref["Q"][same], cfg.bits, cfg.group, cfg.T)
    eq = (Q.cpu().numpy()[cols][same] == refcd["Q"]).mean()
    say(f"  layer loss after CD {float(l_cd.sum()):.6e}; codes equal on {eq:.6f} of sampled entries")
    assert eq >= 0.999


def test_attn_proj_bcd_after_cd(cdq, oracle):
    """Algorithm 2 (k = 2) at the benchmark layer's shape, started from greedy CD's result as in Section 4, T = d_in
    with d_in random partitions: whole layer on the GPU, 24 sampled columns through the oracle (codes and move counts
    equal), loss never above CD's."""
    cfg = inputs.CONFIGS["attn_proj"]
    say(f"{cfg.name}: generating X and Wt")
    X, Wt = inputs.make_layer(cfg)
    Hd = cdq.hessian(x_to_dev(X, cfg.x_dtype))
    H32 = Hd.cpu().numpy()
    del X
    Wd = torch.from_numpy(Wt).cuda()
    scale, zero, Q = cdq.init_rtn(Wd, cfg.bits, cfg.group)
    cdq.greedy_cd(Hd, Wd, scale, zero, Q, cfg.bits, cfg.group, cfg.T)
    q_cd = Q.cpu().numpy().copy()
    l_cd = cdq.loss(Hd, Wd, scale, zero, Q, cfg.group)[0].cpu().numpy()
    T = cfg.d_in
    parts = inputs.make_partitions(T, cfg.d_in, seed=cfg.seed)
    pd = torch.from_numpy(parts).cuda()
    say(f"BCD on the GPU, T={T}")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    out = cdq.bcd(Hd, Wd, scale, zero, Q, cfg.bits, cfg.group, pd)
    torch.cuda.synchronize()
    moves = out["moves"].cpu().numpy()
    say(f"  {1e3 * (time.perf_counter() - t0):.1f} ms, {int(moves.sum())} block moves (max {moves.max()} per column)")
    l_bcd = cdq.loss(Hd, Wd, scale, zero, Q, cfg.group)[0].cpu().numpy()
    assert (moves >= 0).all()
    assert np.all(l_bcd <= l_cd * (1 + 1e-9))
    say(f"  layer loss CD {l_cd.sum():.6e} -> BCD {l_bcd.sum():.6e}")
    assert l_bcd.sum() < l_cd.sum()
    cols = np.sort(np.random.default_rng(3).choice(cfg.d_out, size=24, replace=False))
    say(f"oracle BCD on {len(cols)} sampled columns")
    a, b = scale.cpu().numpy(), zero.cpu().numpy()
    ref = oracle.bcd(H32, Wt[cols], a[cols], b[cols], q_cd[cols], parts, cfg.bits, cfg.group, k=2)
    eq = (Q.cpu().numpy()[cols] == ref["Q"])
    say(f"  codes equal on {eq.mean():.6f} of sampled entries")
    assert eq.all()
    assert np.array_equal(moves[cols], ref["moves"])


@pytest.mark.parametrize("d_in", [24576, 32768, 36864])
def test_wide_layers_against_the_oracle(cdq, oracle, d_in):
    """Above d_in = 16384 the fused loop keeps the Hessian diagonal in LDS (24, 32 or 36 coordinates per lane on 16
    wavefronts); 24576 and 36864 are FFN2 widths of the paper's runtime table.  A few columns, the default launch
    shape, RTN start; the oracle reruns them from the GPU's fp32 H: codes, move counts and the per-column loss
    must match."""
    d_out, n, bits, T = 6, 2048, 3, 96
    say(f"generating X [{n}x{d_in}] on the GPU and Wt [{d_out}x{d_in}]")
    g = torch.Generator(device="cuda")
    g.manual_seed(11)
    Xd = (torch.randn((n, d_in), generator=g, device="cuda") * torch.exp(0.5 * torch.randn(d_in, generator=g, device="cuda"))).to(torch.bfloat16)
    Wt = inputs.make_wt(d_out, d_in, seed=5)
    say("hessian on the GPU")
    Hd = cdq.hessian(Xd)
    del Xd
    Wd = torch.from_numpy(Wt).cuda()
    scale, zero, Q = cdq.init_rtn(Wd, bits, d_in)
    q0 = Q.cpu().numpy().copy()
    say(f"greedy CD on the GPU, T={T}")
    out = cdq.greedy_cd(Hd, Wd, scale, zero, Q, bits, d_in, T)
    st = out["stats"].cpu().numpy()
    per = cdq.loss(Hd, Wd, scale, zero, Q, d_in)[0].cpu().numpy()
    say(f"  moves per column {st[:, 0].tolist()}")
    assert (st[:, 0] > 0).all() and (st[:, 0] <= T).all()
    say("copying H to the host for the oracle")
    H32 = Hd.cpu().numpy()
    a, b = scale.cpu().numpy(), zero.cpu().numpy()
    ref = oracle.greedy_cd(H32, Wt, a, b, q0, bits, d_in, T)
    assert np.array_equal(Q.cpu().numpy(), ref["Q"])
    assert np.array_equal(st[:, 0], ref["moves"])
    np.testing.assert_allclose(per, oracle.loss(H32, Wt, ref["Q"], a, b, d_in), rtol=1e-6)


@pytest.mark.parametrize("d_in,d_out,n_cd,T", [(14336, 2051, 4000, 48), (36864, 2053, 96, 10)])
def test_wide_layer_bcd_against_the_oracle(cdq, oracle, d_in, d_out, n_cd, T):
    """Block CD at FFN2 widths (14336, and 36864, the widest in the paper's runtime table): the wide-layer kernel with 8
    columns per workgroup and a last workgroup of 3 or 5 -- only the 16-bit margins' minimum in LDS, everything else in
    global memory.  Starts from greedy CD's codes (converged at 14336, as the paper starts it; after 96 iterations at
    36864, so that many blocks move); the oracle reruns a sample of the columns from the GPU's fp32 H."""
    n, bits = 2048, 3
    say(f"generating X [{n}x{d_in}] on the GPU and Wt [{d_out}x{d_in}]")
    g = torch.Generator(device="cuda")
    g.manual_seed(13)
    Xd = (torch.randn((n, d_in), generator=g, device="cuda") * torch.exp(0.5 * torch.randn(d_in, generator=g, device="cuda"))
          + torch.randn((n, 1), generator=g, device="cuda")).to(torch.bfloat16)
    Wt = inputs.make_wt(d_out, d_in, seed=6)
    Hd = cdq.hessian(Xd)
    del Xd
    Wd = torch.from_numpy(Wt).cuda()
    scale, zero, Q = cdq.init_rtn(Wd, bits, d_in)
    cdq.greedy_cd(Hd, Wd, scale, zero, Q, bits, d_in, n_cd)
    cols = np.array([0, 7, 1001, 2047, 2048, d_out - 1])
    q_cd = Q.cpu().numpy()[cols].copy()
    parts = inputs.make_partitions(T, d_in, seed=3)
    say(f"BCD on the GPU, T={T}")
    out = cdq.bcd(Hd, Wd, scale, zero, Q, bits, d_in, torch.from_numpy(parts).cuda(), want_G=True)
    moves = out["moves"].cpu().numpy()
    say(f"  block moves: {int(moves.sum())} in all, sampled columns {moves[cols].tolist()}")
    say("copying H to the host for the oracle")
    H32 = Hd.cpu().numpy()
    a, b = scale.cpu().numpy()[cols], zero.cpu().numpy()[cols]
    ref = oracle.bcd(H32, np.ascontiguousarray(Wt[cols]), a, b, q_cd, parts, bits, d_in, k=2)
    assert moves[cols].sum() > 0
    assert np.array_equal(moves[cols], ref["moves"])
    assert np.array_equal(Q.cpu().numpy()[cols], ref["Q"])
    assert np.array_equal(out["G"].cpu().numpy()[cols], ref["G"])


def test_a_column_that_moves_one_coordinate_up_and_down_to_the_end_of_the_budget(cdq, oracle):
    """Where two neighbouring levels of a coordinate have the same loss to within the rounding of the gradient, both moves
    compute to a tiny negative score and the loop of Algorithm 1, run in fp32, alternates between them until the budget
    T is spent (the oracle does the same).  The fused kernel recognises the exact period-2 state and jumps to the end;
    codes, move count and last score must still be those of the oracle, which takes every step.  First seen on the
    Gemma-1 7B FFN2 shape of the layer driver (about one column per layer); here the situation is built on that shape from
    the streamed Hessian's own diagonal, so that it does not depend on the last bits of the sums: every weight on a grid
    point of Eq. (2) except one per column, exactly half way between two levels on a coordinate whose (21/16) H_ii rounds
    up in fp32 by less than a quarter of a unit in the last place."""
    from fractions import Fraction

    from paper_2406_17542_amd.layer import synthetic_chunks, HessianAccumulator
    d_in, d_out, bits = 24576, 6, 3
    say("streaming the Hessian of 655 360 synthetic tokens")
    acc = HessianAccumulator(d_in, "cuda")
    it = iter(synthetic_chunks(320 * 2048, d_in, 65536, seed=3))
    cur = next(it)
    while cur is not None:
        nxt = next(it, None)
        acc.add(cur, last=nxt is None, lambda_rel=0.01)
        cur = nxt
    Hd = acc.H
    hdiag = torch.diagonal(Hd).cpu().numpy()
    good = []
    for i in range(2, d_in):
        p = Fraction(21, 16) * Fraction(float(hdiag[i]))
        f32 = np.float32(float(p))
        if 0 < Fraction(float(f32)) - p < Fraction(float(np.spacing(f32))) / 4:
            good.append(i)
        if len(good) == d_out:
            break
    assert len(good) == d_out
    r = np.random.default_rng(4)
    Wt = (np.float32(1.3125) * r.integers(0, 8, (d_out, d_in))).astype(np.float32)
    Wt[:, 0], Wt[:, 1] = 0.0, 9.1875
    for j in range(d_out):
        Wt[j, good[j]] = 3.28125
    Wd = torch.from_numpy(Wt).cuda()
    scale, zero, Q = cdq.init_rtn(Wd, bits, d_in)
    assert torch.all(scale == 1.3125) and torch.all(zero == 0)
    q0 = Q.cpu().numpy().copy()
    shape = cdq.greedy_cd_shape(3072, d_in, d_in)          # the launch shape of the whole layer (16 wavefronts, 24 per lane)
    say(f"greedy CD on the GPU, T = d_in, launch shape {shape}")
    cdq.greedy_cd(Hd, Wd, scale, zero, Q.clone(), bits, d_in, 1, waves_per_column=shape[0], elems_per_lane=shape[1])     # first use of this kernel
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    out = cdq.greedy_cd(Hd, Wd, scale, zero, Q, bits, d_in, d_in, waves_per_column=shape[0], elems_per_lane=shape[1])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    say(f"  {dt:.3f} s")
    st = out["stats"].cpu().numpy()
    assert np.all(st[:, 0] == d_in), "every column of the case alternates to the end of its budget"
    assert dt < 0.1, "the kernel should have jumped over the periodic part (taking every step needs about 0.2 s)"
    say("copying H to the host; the oracle takes every step")
    H32 = Hd.cpu().numpy()
    a, b = scale.cpu().numpy(), zero.cpu().numpy()
    ref = oracle.greedy_cd(H32, Wt, a, b, q0, bits, d_in, d_in)
    assert np.array_equal(st[:, 0], ref["moves"])
    assert np.array_equal(Q.cpu().numpy(), ref["Q"])
    # an odd budget ends in the other state of the pair
    Q2 = torch.from_numpy(q0[:1].copy()).cuda()
    out2 = cdq.greedy_cd(Hd, Wd[:1].contiguous(), scale[:1].contiguous(), zero[:1].contiguous(), Q2, bits, d_in, d_in - 1,
                         waves_per_column=shape[0], elems_per_lane=shape[1])
    ref2 = oracle.greedy_cd(H32, Wt[:1], a[:1], b[:1], q0[:1], bits, d_in, d_in - 1)
    assert np.array_equal(out2["stats"].cpu().numpy()[:, 0], ref2["moves"]) and ref2["moves"][0] == d_in - 1
    assert np.array_equal(Q2.cpu().numpy(), ref2["Q"])
    assert not np.array_equal(ref2["Q"], ref["Q"][:1])
