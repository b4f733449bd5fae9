"""The two scorers of the fused greedy-CD loop (Algorithm 1, the arg-min step), modelled in numpy fp32 and compared on
adversarial inputs, on the CPU.

The loop scores, per coordinate, only the level nearest to the minimiser rf = q - 2g / (2 a H_ii) of the score parabola
("nearest-level scorer"), and redoes an iteration with the two-level scorer (floor and ceil of rf, both by the canonical
formula s = delta * fma(delta, H_ii, 2g), delta = a (r - q): the same winner as a scan of all levels) when the winning
coordinate is flagged -- rf within 2^-9 of a half-integer -- or no move was found.  What include/cdq.h states about the
difference between the two is pinned here:
  * a coordinate that is not flagged is scored identically by both (same level, same score bits);
  * the two can pick different levels for a coordinate only if its exact minimiser lies within 2^-15 of a half-integer,
    and the canonical scores of the two levels then differ by at most 2^-15 a^2 H_ii + 2^-21 |s|.
So a move of the nearest-level scorer can differ from Algorithm 1's arg-min only through a flagged coordinate that is NOT
the winner and whose better level would have beaten the winner by less than that amount."""
import numpy as np

F = np.float32


def fma(a, b, c):
    # fp32 fused multiply-add: the product of two fp32 values is exact in fp64
    return (a.astype(np.float64) * b.astype(np.float64) + c.astype(np.float64)).astype(np.float32)


def canonical_score(a, h, g2, u):
    d = (a * u).astype(np.float32)
    return (d * fma(d, h, g2)).astype(np.float32)


def nearest_level(a, h, g2, q, top, cinv):
    rf = fma(-g2, cinv, q)
    rn = np.clip(np.rint(rf), 0, top).astype(np.float32)
    frac = rf - np.floor(rf)
    flag = np.abs(frac - F(0.5)) < F(1.0 / 512.0)
    return rn, canonical_score(a, h, g2, rn - q), flag


def two_levels(a, h, g2, q, top, cinv):
    rf = np.clip(fma(-g2, cinv, q), 0, top).astype(np.float32)
    r0, r1 = np.floor(rf), np.ceil(rf)
    s0, s1 = canonical_score(a, h, g2, r0 - q), canonical_score(a, h, g2, r1 - q)
    take1 = s1 < s0                                   # equal scores keep the lower level
    return np.where(take1, r1, r0).astype(np.float32), np.where(take1, s1, s0).astype(np.float32)


def adversarial_cases(seed, n, bits):
    """Coordinates whose minimiser sits at a half-integer plus a tiny offset, from exactly on it to well outside the flag
    window, with the reciprocal of the curvature off by up to an ulp either way."""
    r = np.random.default_rng(seed)
    top = F((1 << bits) - 1)
    a = np.exp(r.uniform(-6, 2, n)).astype(np.float32)
    h = np.exp(r.uniform(-3, 12, n)).astype(np.float32)
    q = r.integers(0, int(top) + 1, n).astype(np.float32)
    k = r.integers(-1, int(top) + 1, n).astype(np.float64)                     # midpoint k + 1/2, also just outside the grid
    off = np.where(r.random(n) < 0.2, 0.0, r.choice([-1.0, 1.0], n) * np.exp2(r.uniform(-26, -8, n)))
    target = k + 0.5 + off
    curv = 2.0 * a.astype(np.float64) * h.astype(np.float64)
    g2 = (-(target - q.astype(np.float64)) * curv).astype(np.float32)
    g2 = np.nextafter(g2, np.where(r.random(n) < 0.5, F(np.inf), F(-np.inf))) if seed % 2 else g2
    cinv = (1.0 / (2.0 * a * h).astype(np.float32).astype(np.float64)).astype(np.float32)
    ulps = r.integers(-1, 2, n)
    cinv = np.where(ulps > 0, np.nextafter(cinv, F(np.inf)), np.where(ulps < 0, np.nextafter(cinv, F(0)), cinv)).astype(np.float32)
    return a, h, g2, q, top, cinv


def test_scorers_differ_only_within_rounding_of_a_half_integer_and_by_a_bounded_score():
    n_diff = 0
    for bits in (2, 3, 4):
        for seed in range(6):
            a, h, g2, q, top, cinv = adversarial_cases(100 * bits + seed, 200_000, bits)
            rn, s_fast, flag = nearest_level(a, h, g2, q, top, cinv)
            re, s_exact = two_levels(a, h, g2, q, top, cinv)
            # the exact minimiser of the parabola, in fp64, clamped like the kernels clamp it
            rf_true = np.clip(q.astype(np.float64) - g2.astype(np.float64) / (2.0 * a.astype(np.float64) * h.astype(np.float64)), 0, float(top))
            dist = np.abs(rf_true - np.floor(rf_true) - 0.5)
            differ = (rn != re) & ((s_fast < 0) | (s_exact < 0))               # levels with a score >= 0 are no moves for either
            n_diff += int(differ.sum())
            # not flagged: same level and the same score, bit for bit
            calm = ~flag
            same_move = (rn == re) | ((s_fast >= 0) & (s_exact >= 0))
            assert same_move[calm].all()
            both = calm & (rn == re) & (s_exact < 0)                       # a score of zero (either sign) is no move
            assert np.array_equal(s_fast[both].view(np.uint32), s_exact[both].view(np.uint32))
            # flagged and different: only within 2^-15 of the half-integer (where the fp32 scores of the two levels round
            # to within a few units of each other), and the scores are that close
            assert flag[differ].all()
            assert (dist[differ] <= 2.0 ** -15).all(), float(dist[differ].max())
            a2h = a.astype(np.float64) ** 2 * h.astype(np.float64)
            gap = np.abs(s_fast.astype(np.float64) - s_exact.astype(np.float64))
            bound = 2.0 ** -15 * a2h + 2.0 ** -21 * np.abs(s_exact.astype(np.float64))
            assert (gap[differ] <= bound[differ]).all(), float((gap[differ] / bound[differ]).max())
    assert n_diff > 1000, "the cases should make the two scorers disagree often enough to mean something"


def test_two_level_scorer_is_the_scan_of_all_levels():
    """floor / ceil of the clamped minimiser against a scan of all 2^c levels with the canonical formula: same score, and
    the same level wherever that score is a move (negative)."""
    for bits in (2, 3, 4):
        a, h, g2, q, top, cinv = adversarial_cases(7 + bits, 100_000, bits)
        r2, s2 = two_levels(a, h, g2, q, top, cinv)
        best_s = np.full(len(a), np.inf, np.float32)
        best_r = np.zeros(len(a), np.float32)
        for lev in range(int(top) + 1):                                       # ascending: the first strict minimum wins ties
            s = canonical_score(a, h, g2, F(lev) - q)
            better = s < best_s
            best_s = np.where(better, s, best_s)
            best_r = np.where(better, F(lev), best_r)
        move = best_s < 0
        assert np.array_equal(s2[move].view(np.uint32), best_s[move].view(np.uint32))
        assert np.array_equal(r2[move], best_r[move])
        assert (s2[~move] >= 0).all()
