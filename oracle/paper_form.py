"""Literal fp64 transcriptions of the paper's own formulations.  TEST INFRASTRUCTURE ONLY.

These follow the paper's notation (code space: the gradient is taken with
respect to the integer codes q, the score is u^2 H_ii + u g_i) rather than the
weight-space form the C oracle and the HIP library use.  They exist so the
C oracle can be pinned against an independent statement of the same method:
the two forms must select the same sequence of moves.

One column at a time, numpy fp64, tiny sizes only.
"""
from __future__ import annotations

import itertools

import numpy as np


def layer_loss(X, w, a, b, q):
    """Eq. (1): ||X (w - a q - b)||_2^2 for one column; a, b scalars or per-coordinate
    vectors (the sub-channel form, appendix 'CDQuant for sub-channel quantization')."""
    r = X @ (w - a * q - b)
    return float(r @ r)


def greedy_cd_code_space(X, w, a, b, q0, T, bits):
    """Algorithm 1, step by step as printed: H = X^T X, g = 2H(q0 - (w-b)/a),
    then T times: arg-min over (i, r) of (r-q_i)^2 H_ii + (r-q_i) g_i, gradient
    update with column i* of H, code update.  The table of scores contains
    r = q_i (score 0); when its minimum is not negative the step is a no-op, so
    the loop stops there.  Returns (q_T, list of (i*, r*, score))."""
    X = np.asarray(X, np.float64)
    H = X.T @ X
    q = np.asarray(q0, np.float64).copy()
    g = 2.0 * H @ (q - (w - b) / a)
    levels = np.arange(1 << bits, dtype=np.float64)
    moves = []
    for _ in range(T):
        u = levels[None, :] - q[:, None]
        score = u * u * np.diag(H)[:, None] + u * g[:, None]
        flat = int(np.argmin(score))            # first minimum in (i, r) order
        i, r = divmod(flat, 1 << bits)
        if not score[i, r] < 0.0:
            break
        g = g + 2.0 * (r - q[i]) * H[:, i]
        moves.append((i, r, float(score[i, r])))
        q[i] = r
    return q.astype(np.int64), moves


def greedy_cd_sub_channel(X, w, a_vec, b_vec, q0, T, bits):
    """Algorithm 4: rescale X~ = X diag(a), w~ = w / a, b~ = b / a (as the
    appendix text defines them) and run Algorithm 1 on the rescaled problem with
    unit scale.  Scores returned are those of the rescaled problem, which equal
    the true loss change."""
    a_vec = np.asarray(a_vec, np.float64)
    Xt = np.asarray(X, np.float64) * a_vec[None, :]
    return greedy_cd_code_space(Xt, np.asarray(w, np.float64) / a_vec, 1.0,
                                np.asarray(b_vec, np.float64) / a_vec, q0, T, bits)


def brute_force_best(X, w, a, b, bits):
    """Global minimum of Eq. (1) over all codes, by enumeration (d_in <= 8 or so)."""
    d = X.shape[1]
    best, best_q = np.inf, None
    for code in itertools.product(range(1 << bits), repeat=d):
        q = np.array(code, np.float64)
        v = layer_loss(X, w, a, b, q)
        if v < best:
            best, best_q = v, q
    return best, best_q.astype(np.int64)


def clip_grid(w, bits, gamma):
    """Eq. (2): a = gamma (max w - min w) / (2^c - 1), b = min w,
    q = clamp(round((w - b)/a), 0, 2^c - 1).  fp64, one group."""
    w = np.asarray(w, np.float64)
    a = gamma * (w.max() - w.min()) / ((1 << bits) - 1)
    b = w.min()
    q = np.clip(np.rint((w - b) / a), 0, (1 << bits) - 1)
    return a, b, q.astype(np.int64)


def owc_cd_paper_form(X, w, bits, group, gammas, T):
    """Algorithm 3 in the paper's notation (fp64): residual table Delta(i, beta) = w - a q - b per
    group and grid point, every group starting at the last grid point (gamma = 1), H = X^T X,
    v = 2 H (a q + b - w)  [the sign that makes the score the loss change; the box prints a minus],
    then T times: arg-min over (i, beta) of
    (Delta(i,gamma_i) - Delta(i,beta))^T H_ii (...) + v_i^T (Delta(i,gamma_i) - Delta(i,beta)),
    update v and gamma_i.  Returns (list of chosen grid indices per group, list of moves)."""
    X = np.asarray(X, np.float64)
    w = np.asarray(w, np.float64)
    d = len(w)
    n_grp = d // group
    H = X.T @ X
    delta = np.empty((len(gammas), d))
    for k, beta in enumerate(gammas):
        for i in range(n_grp):
            sl = slice(i * group, (i + 1) * group)
            a, b, q = clip_grid(w[sl], bits, float(beta))
            delta[k, sl] = w[sl] - a * q - b
    cur = [len(gammas) - 1] * n_grp
    e = -delta[-1].copy()                     # a q + b - w
    v = 2.0 * H @ e
    moves = []
    for _ in range(T):
        best = (0.0, -1, -1)
        for i in range(n_grp):
            sl = slice(i * group, (i + 1) * group)
            for k in range(len(gammas)):
                if k == cur[i]:
                    continue
                diff = delta[cur[i], sl] - delta[k, sl]
                s = diff @ H[sl, sl] @ diff + v[sl] @ diff
                if s < best[0]:
                    best = (s, i, k)
        if best[1] < 0:
            break
        s, i, k = best
        sl = slice(i * group, (i + 1) * group)
        diff = delta[cur[i], sl] - delta[k, sl]
        v = v + 2.0 * H[:, sl] @ diff
        cur[i] = k
        moves.append((i, k, s))
    return cur, moves


def bcd_code_space(X, w, a, b, q0, parts, bits, k=2):
    """Algorithm 2 as printed (fp64, code space): g = 2H(q0 - (w-b)/a); per iteration, for the given
    partition into blocks of k, arg-min over blocks i and level tuples r of
    (r - q_i)^T H_ii (r - q_i) + (r - q_i)^T g_i, then g += 2 H[:, block] (r* - q_block) and the
    codes of the block are replaced.  A minimum that is not negative changes nothing.
    Returns (q_T, list of (t, block, tuple of levels, score))."""
    X = np.asarray(X, np.float64)
    H = X.T @ X
    q = np.asarray(q0, np.float64).copy()
    g = 2.0 * H @ (q - (np.asarray(w, np.float64) - b) / a)
    tuples = np.array(list(itertools.product(range(1 << bits), repeat=k)), np.float64)     # first member outermost
    moves = []
    for t, part in enumerate(np.asarray(parts)):
        best = (0.0, -1, None)
        for blk in range(len(part) // k):
            idx = part[blk * k:(blk + 1) * k]
            u = tuples - q[idx][None, :]
            sc = np.einsum("tm,mn,tn->t", u, H[np.ix_(idx, idx)], u) + u @ g[idx]
            m = int(np.argmin(sc))
            if sc[m] < best[0]:
                best = (float(sc[m]), blk, tuples[m].copy())
        if best[1] < 0:
            continue
        s, blk, r = best
        idx = part[blk * k:(blk + 1) * k]
        g = g + 2.0 * H[:, idx] @ (r - q[idx])
        q[idx] = r
        moves.append((t, blk, tuple(int(x) for x in r), s))
    return q.astype(np.int64), moves


def bcd_sub_channel(X, w, a_vec, b_vec, q0, parts, bits, k=2):
    """Algorithm 5: Algorithm 2 on X~ = X diag(a), w~ = w / a, b~ = b / a with unit scale."""
    a_vec = np.asarray(a_vec, np.float64)
    return bcd_code_space(np.asarray(X, np.float64) * a_vec[None, :], np.asarray(w, np.float64) / a_vec, 1.0,
                          np.asarray(b_vec, np.float64) / a_vec, q0, parts, bits, k)
