"""The inequalities behind the block-CD kernels' pair skipping, checked on the CPU in plain numpy.

The kernels leave a pair (i, k) unscored when a bound says that none of its moves lowers the loss
(Algorithm 2's score for a block of two, weight-space form).  These tests evaluate the bound and the
fp32 scores independently of the library: whenever the bound holds, every level pair of the pair must
have a non-negative score computed exactly as the kernels and the oracle compute it.  They also mirror
the 16-bit fixed-point form of the test that the multi-column kernel uses and check that it never
accepts a pair the real-valued test rejects.
"""
import numpy as np

TAU = np.float32(2.0 ** -14)
f32 = np.float32


def fma32(a, b, c):
    """fp32 fused multiply-add: the product and sum are exact in fp64 for fp32 inputs of this size."""
    return f32(np.float64(a) * np.float64(b) + np.float64(c))


def pair_scores(a_i, a_k, q_i, q_k, g2_i, g2_k, h_ii, h_kk, h2_ik, levels):
    """All level pairs' scores s = fma(di*dk, 2H_ik, di*fma(di,H_ii,2g_i) + dk*fma(dk,H_kk,2g_k)) in fp32."""
    out = np.empty((levels, levels), np.float32)
    for ri in range(levels):
        di = f32(a_i * f32(ri - q_i))
        si = f32(di * fma32(di, h_ii, g2_i))
        for rk in range(levels):
            dk = f32(a_k * f32(rk - q_k))
            sk = f32(dk * fma32(dk, h_kk, g2_k))
            out[ri, rk] = fma32(f32(di * dk), h2_ik, f32(si + sk))
    return out


def random_case(rng, near_optimum):
    """One pair: a positive definite 2x2 block, grid steps, codes and gradients; near_optimum puts the
    gradients close to (and on both sides of) the edge of what a single-coordinate move can improve."""
    levels = int(rng.choice([4, 8, 16]))
    h_ii, h_kk = f32(rng.uniform(0.5, 50.0)), f32(rng.uniform(0.5, 50.0))
    rho = rng.uniform(0.0, 0.95) * rng.choice([1.0, 1.0, 0.05])
    h_ik = f32(rng.choice([-1.0, 1.0]) * rho * np.sqrt(np.float64(h_ii) * np.float64(h_kk)))
    a_i, a_k = f32(rng.uniform(0.01, 2.0)), f32(rng.uniform(0.01, 2.0))
    q_i, q_k = int(rng.integers(levels)), int(rng.integers(levels))
    if near_optimum:
        u_i, u_k = rng.uniform(0.0, 1.02), rng.uniform(0.0, 1.02)
        if rng.random() < 0.3:
            u_i = 1.0 - rng.uniform(0.0, 4e-4)
    else:
        u_i, u_k = rng.uniform(0.0, 3.0), rng.uniform(0.0, 3.0)
    g2_i = f32(rng.choice([-1.0, 1.0]) * u_i * np.float64(h_ii) * np.float64(a_i))
    g2_k = f32(rng.choice([-1.0, 1.0]) * u_k * np.float64(h_kk) * np.float64(a_k))
    return levels, a_i, a_k, q_i, q_k, g2_i, g2_k, h_ii, h_kk, f32(2.0) * h_ik


def u_of(g2, h, a):
    return f32(np.abs(g2)) / f32(h * a)


def rho_of(h2_ik, h_ii, h_kk):
    return f32(f32(f32(0.5) * np.abs(h2_ik)) / np.sqrt(h_ii)) / np.sqrt(h_kk)


def test_sum_form_of_the_bound_never_skips_an_improving_pair():
    """One-column kernel: u_i, u_k <= 1 - rho - tau  =>  no level pair has a negative fp32 score."""
    rng = np.random.default_rng(1)
    skipped = 0
    for n in range(6000):
        lv, a_i, a_k, q_i, q_k, g2_i, g2_k, h_ii, h_kk, h2 = random_case(rng, near_optimum=n % 2 == 0)
        thr = f32(1.0) - rho_of(h2, h_ii, h_kk) - TAU
        if u_of(g2_i, h_ii, a_i) <= thr and u_of(g2_k, h_kk, a_k) <= thr:
            skipped += 1
            assert pair_scores(a_i, a_k, q_i, q_k, g2_i, g2_k, h_ii, h_kk, h2, lv).min() >= 0.0
    assert skipped > 500


def v16(g2, h, a):
    """1 - u - tau in units of 2^-16, rounded down by more than one unit (0: never skip)."""
    u = u_of(g2, h, a)
    return int(65530 - int(f32(u * f32(65536.0)))) if 0.0 <= u < f32(0.99985) else 0


def r16(h2_ik, h_ii, h_kk):
    """rho^2 in units of 2^-16, rounded up by more than one unit (65535: never skip)."""
    if not (h_ii > 0 and h_kk > 0):
        return 65535
    rho = rho_of(h2_ik, h_ii, h_kk)
    r2 = f32(rho * rho)
    return int(f32(r2 * f32(65536.0))) + 2 if r2 < f32(0.99) else 65535


def test_product_form_of_the_bound_never_skips_an_improving_pair():
    """Multi-column kernel: (1-u_i-tau)(1-u_k-tau) >= rho^2 with both factors >= 0, in its 16-bit form
    (v_i v_k) >> 16 >= R.  The fixed-point test must imply the real-valued one, and a skipped pair must
    have no negative fp32 score.  The product form must also skip every pair the sum form skips."""
    rng = np.random.default_rng(2)
    skipped = both = 0
    for n in range(8000):
        lv, a_i, a_k, q_i, q_k, g2_i, g2_k, h_ii, h_kk, h2 = random_case(rng, near_optimum=n % 2 == 0)
        vi, vk, R = v16(g2_i, h_ii, a_i), v16(g2_k, h_kk, a_k), r16(h2, h_ii, h_kk)
        quiet = ((vi * vk) >> 16) >= R
        ui, uk = np.float64(u_of(g2_i, h_ii, a_i)), np.float64(u_of(g2_k, h_kk, a_k))
        rho = np.float64(rho_of(h2, h_ii, h_kk))
        if quiet:
            skipped += 1
            fi, fk = 1.0 - ui - float(TAU), 1.0 - uk - float(TAU)
            assert fi >= 0.0 and fk >= 0.0 and fi * fk >= rho * rho
            assert pair_scores(a_i, a_k, q_i, q_k, g2_i, g2_k, h_ii, h_kk, h2, lv).min() >= 0.0
        thr = 1.0 - rho - 2.0 ** -10                    # the sum form with a margin that covers the 16-bit roundings
        if ui <= thr and uk <= thr:
            both += 1
            assert quiet
    assert skipped > 700 and both > 300


def test_margin_tau_covers_the_rounding_of_the_scores():
    """Pairs exactly on the edge of the real-valued bound (product equal to rho^2 with tau = 0) can have
    fp32 scores a rounding error below zero; with tau = 2^-14 the smallest score of a skipped pair stays
    above tau/2 times the curvature terms, i.e. far from zero."""
    rng = np.random.default_rng(3)
    worst = np.inf
    for _ in range(4000):
        lv, a_i, a_k, q_i, q_k, g2_i, g2_k, h_ii, h_kk, h2 = random_case(rng, near_optimum=True)
        vi, vk, R = v16(g2_i, h_ii, a_i), v16(g2_k, h_kk, a_k), r16(h2, h_ii, h_kk)
        if ((vi * vk) >> 16) < R:
            continue
        s = pair_scores(a_i, a_k, q_i, q_k, g2_i, g2_k, h_ii, h_kk, h2, lv).astype(np.float64)
        for ri in range(lv):
            for rk in range(lv):
                if ri == q_i and rk == q_k:
                    continue
                x2 = (float(a_i) * (ri - q_i)) ** 2 * float(h_ii)
                y2 = (float(a_k) * (rk - q_k)) ** 2 * float(h_kk)
                worst = min(worst, s[ri, rk] / (x2 + y2))
    assert worst >= 0.5 * float(TAU)


def test_division_free_product_form_never_skips_an_improving_pair():
    """Wide-layer kernel: the product form in fp32 without divisions, (w_i (1-tau) - |2g_i|)(w_k (1-tau) - |2g_k|) >=
    rho^2 w_i w_k with w = H a and both factors >= 0.  A skipped pair must have no negative fp32 score."""
    rng = np.random.default_rng(4)
    skipped = 0
    for n in range(8000):
        lv, a_i, a_k, q_i, q_k, g2_i, g2_k, h_ii, h_kk, h2 = random_case(rng, near_optimum=n % 2 == 0)
        rho = rho_of(h2, h_ii, h_kk)
        r2 = f32(rho * rho)
        wi, wk = f32(h_ii * a_i), f32(h_kk * a_k)
        one_tau = f32(f32(1.0) - TAU)
        mi = f32(np.float64(wi) * np.float64(one_tau) - np.float64(abs(g2_i)))
        mk = f32(np.float64(wk) * np.float64(one_tau) - np.float64(abs(g2_k)))
        if mi >= 0 and mk >= 0 and f32(mi * mk) >= f32(f32(r2 * wi) * wk):
            skipped += 1
            assert pair_scores(a_i, a_k, q_i, q_k, g2_i, g2_k, h_ii, h_kk, h2, lv).min() >= 0.0
    assert skipped > 700


def test_a_coordinate_held_at_the_end_of_its_grid_counts_with_u_zero():
    """All three kernels: a coordinate whose code is 0 (or the top level) while 2g asks for a step further down
    (up) has only moves with delta * 2g >= 0; the bound then holds with u = 0 for it.  Pairs skipped with that
    substitution, and not without it, must still have no negative fp32 score."""
    rng = np.random.default_rng(5)
    extra = 0
    for n in range(12000):
        lv, a_i, a_k, q_i, q_k, g2_i, g2_k, h_ii, h_kk, h2 = random_case(rng, near_optimum=n % 4 != 0)
        q_i = int(rng.choice([0, lv - 1]))
        if n % 3 == 0:
            q_k = int(rng.choice([0, lv - 1]))
        if n % 2 == 0:                                  # strong outward gradients: the plain test would never skip these
            g2_i = f32(g2_i * f32(rng.uniform(1.0, 30.0)))

        def u_eff(g2, h, a, q):
            held = a > 0 and ((g2 > 0 and q == 0) or (g2 < 0 and q == lv - 1))
            return np.float64(0.0) if held else np.float64(u_of(g2, h, a))

        rho = np.float64(rho_of(h2, h_ii, h_kk))
        fi, fk = 1.0 - u_eff(g2_i, h_ii, a_i, q_i) - float(TAU), 1.0 - u_eff(g2_k, h_kk, a_k, q_k) - float(TAU)
        pi, pk = 1.0 - np.float64(u_of(g2_i, h_ii, a_i)) - float(TAU), 1.0 - np.float64(u_of(g2_k, h_kk, a_k)) - float(TAU)
        if fi >= 0 and fk >= 0 and fi * fk >= rho * rho * (1.0 + 1e-4):
            if not (pi >= 0 and pk >= 0 and pi * pk >= rho * rho):
                extra += 1
            assert pair_scores(a_i, a_k, q_i, q_k, g2_i, g2_k, h_ii, h_kk, h2, lv).min() >= 0.0
    assert extra > 1000
