/*
 * CPU oracle for the CDQuant hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, scalar C that states what the path computes, written from the
 * paper (arXiv 2406.17542).  Nothing in the product path may call it: only
 * tests, the smoke check and the benchmark's cpu_baseline leg do.  It shares
 * no code, header, table or helper with the HIP library.
 *
 * Conventions (weight space, one Hessian for every output column):
 *   Wt, Q        [d_out][d_in] row-major: row j is output column j of the
 *                paper's W (Section 3, Notation), so every row is one
 *                independent problem of the form of Eq. (1).
 *   scale, zero  [d_out][d_in/group]: the paper's a and b, one pair per group
 *                of `group` consecutive input coordinates (Section 3.2);
 *                group == d_in is per-channel quantization.
 *   e = a*q + b - w   (the quantization residual of one column)
 *   g = H e           (half the gradient of Eq. (1) with respect to a*q)
 *
 * The paper's Algorithm 1 keeps g_p = 2H(q - (w-b)/a) = (2/a) H e and scores a
 * move of coordinate i to level r by u^2 H_ii + u g_p,i with u = r - q_i.
 * Multiplying by the positive per-column constant a^2 gives
 *   s(i,r) = delta^2 H_ii + 2 delta g_i,  delta = a u,
 * which is the exact change of the loss of Eq. (1).  With per-group scales the
 * appendix's Algorithm 4 rescales X by diag(a); substituting H~ = D_a H D_a
 * into its score gives the same s(i,r) with delta = a_grp(i) u.  So one routine
 * serves Algorithm 1 and Algorithm 4.
 *
 * Readings where the paper is silent:
 *   - arg-min ties: smallest score, then smallest i, then smallest r.
 *   - a move is committed only if its score is < 0; otherwise the column has
 *     reached a coordinate-wise optimum and stops (later iterations are no-ops).
 *   - "canonical" fp32 arithmetic of the *_f32 routines, so that another fp32
 *     implementation can reproduce them bit for bit:
 *         e_i   = fmaf(a, (float)q_i, b) - w_i
 *         g_i   = (float) sum_k (double)H_ik * (double)e_k     (k ascending)
 *         delta = a * (float)(r - q_i)
 *         s     = delta * fmaf(delta, H_ii, 2*g_i)
 *         g_k  <- fmaf(delta*, H[i*][k], g_k)
 *
 * Pins (tests/test_oracle_*.py): brute force over all codes on tiny layers,
 * score == recomputed loss change, monotone loss, diagonal-H closed form,
 * agreement with a literal code-space transcription of Algorithms 1 and 4
 * (oracle/paper_form.py), ||XE||^2 == tr(E^T H E).  The paper prints no worked
 * numeric example, so no value here is pinned to a printed number.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

/* ---- residual e = a q + b - w  (Section 3, Notation; groups: Section 3.2) ---- */

void cdqo_residual_f32(const float *Wt, const uint8_t *Q, const float *scale, const float *zero,
                       int64_t d_out, int64_t d_in, int64_t group, float *E)
{
    const int64_t n_grp = d_in / group;
    for (int64_t j = 0; j < d_out; ++j)
        for (int64_t i = 0; i < d_in; ++i) {
            const float a = scale[j * n_grp + i / group];
            const float b = zero[j * n_grp + i / group];
            E[j * d_in + i] = fmaf(a, (float)Q[j * d_in + i], b) - Wt[j * d_in + i];
        }
}

void cdqo_residual_f64(const double *Wt, const uint8_t *Q, const double *scale, const double *zero,
                       int64_t d_out, int64_t d_in, int64_t group, double *E)
{
    const int64_t n_grp = d_in / group;
    for (int64_t j = 0; j < d_out; ++j)
        for (int64_t i = 0; i < d_in; ++i) {
            const double a = scale[j * n_grp + i / group];
            const double b = zero[j * n_grp + i / group];
            E[j * d_in + i] = a * (double)Q[j * d_in + i] + b - Wt[j * d_in + i];
        }
}

/* ---- g = H e for every column (Algorithm 1, "Compute gradient", rescaled) ---- */

void cdqo_gradient_f32(const float *H, const float *E, int64_t d_out, int64_t d_in, float *G)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < d_out; ++j)
        for (int64_t i = 0; i < d_in; ++i) {
            double acc = 0.0;
            for (int64_t k = 0; k < d_in; ++k)
                acc += (double)H[i * d_in + k] * (double)E[j * d_in + k];
            G[j * d_in + i] = (float)acc;
        }
}

void cdqo_gradient_f64(const double *H, const double *E, int64_t d_out, int64_t d_in, double *G)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < d_out; ++j)
        for (int64_t i = 0; i < d_in; ++i) {
            double acc = 0.0;
            for (int64_t k = 0; k < d_in; ++k)
                acc += H[i * d_in + k] * E[j * d_in + k];
            G[j * d_in + i] = acc;
        }
}

/* ---- loss_j = e_j^T H e_j  (Eq. (1) written with H = X^T X) ---- */

void cdqo_loss_f64(const double *H, const double *E, int64_t d_out, int64_t d_in, double *loss)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < d_out; ++j) {
        double tot = 0.0;
        for (int64_t i = 0; i < d_in; ++i) {
            double acc = 0.0;
            for (int64_t k = 0; k < d_in; ++k)
                acc += H[i * d_in + k] * E[j * d_in + k];
            tot += E[j * d_in + i] * acc;
        }
        loss[j] = tot;
    }
}

/* ---- greedy coordinate descent (Algorithm 1; Algorithm 4 for groups) ----
 *
 * G holds g = H e of the initial codes on entry and of the final codes on
 * exit; Q holds q_0 on entry and q_T on exit.  Per column: moves[j] = number
 * of committed moves, converged[j] = 1 if the column stopped because no move
 * lowers the loss.  If trace_cap > 0 the committed moves of column j are
 * recorded in trace_i/trace_r/trace_s[j*trace_cap + m] for m < trace_cap.
 */

void cdqo_greedy_cd_f32(const float *H, const float *scale, uint8_t *Q, float *G,
                        int64_t d_out, int64_t d_in, int bits, int64_t group, int64_t T,
                        int32_t *moves, int32_t *converged,
                        int32_t *trace_i, int32_t *trace_r, float *trace_s, int64_t trace_cap)
{
    const int levels = 1 << bits;
    const int64_t n_grp = d_in / group;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t j = 0; j < d_out; ++j) {
        uint8_t *q = Q + j * d_in;
        float *g = G + j * d_in;
        const float *a = scale + j * n_grp;
        int32_t n_moves = 0, done = 0;
        for (int64_t t = 0; t < T; ++t) {
            /* arg-min over every coordinate and every level (Algorithm 1, the arg-min step) */
            float best_s = 0.0f;
            int64_t best_i = -1;
            int best_r = -1;
            for (int64_t i = 0; i < d_in; ++i) {
                const float ai = a[i / group];
                const float hii = H[i * d_in + i];
                const float two_g = 2.0f * g[i];
                for (int r = 0; r < levels; ++r) {
                    if (r == (int)q[i]) continue;
                    const float delta = ai * (float)(r - (int)q[i]);
                    const float s = delta * fmaf(delta, hii, two_g);
                    if (s < best_s) { best_s = s; best_i = i; best_r = r; }
                }
            }
            if (best_i < 0) { done = 1; break; }          /* coordinate-wise optimum */
            const float delta = a[best_i / group] * (float)(best_r - (int)q[best_i]);
            if (n_moves < trace_cap) {
                trace_i[j * trace_cap + n_moves] = (int32_t)best_i;
                trace_r[j * trace_cap + n_moves] = best_r;
                trace_s[j * trace_cap + n_moves] = best_s;
            }
            q[best_i] = (uint8_t)best_r;                   /* code update */
            const float *hrow = H + best_i * d_in;         /* H symmetric: row = column */
            for (int64_t k = 0; k < d_in; ++k)             /* gradient update */
                g[k] = fmaf(delta, hrow[k], g[k]);
            ++n_moves;
        }
        moves[j] = n_moves;
        converged[j] = done;
    }
}

void cdqo_greedy_cd_f64(const double *H, const double *scale, uint8_t *Q, double *G,
                        int64_t d_out, int64_t d_in, int bits, int64_t group, int64_t T,
                        int32_t *moves, int32_t *converged,
                        int32_t *trace_i, int32_t *trace_r, double *trace_s, int64_t trace_cap)
{
    const int levels = 1 << bits;
    const int64_t n_grp = d_in / group;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t j = 0; j < d_out; ++j) {
        uint8_t *q = Q + j * d_in;
        double *g = G + j * d_in;
        const double *a = scale + j * n_grp;
        int32_t n_moves = 0, done = 0;
        for (int64_t t = 0; t < T; ++t) {
            double best_s = 0.0;
            int64_t best_i = -1;
            int best_r = -1;
            for (int64_t i = 0; i < d_in; ++i) {
                const double ai = a[i / group];
                const double hii = H[i * d_in + i];
                for (int r = 0; r < levels; ++r) {
                    if (r == (int)q[i]) continue;
                    const double delta = ai * (double)(r - (int)q[i]);
                    const double s = delta * (delta * hii + 2.0 * g[i]);
                    if (s < best_s) { best_s = s; best_i = i; best_r = r; }
                }
            }
            if (best_i < 0) { done = 1; break; }
            const double delta = a[best_i / group] * (double)(best_r - (int)q[best_i]);
            if (n_moves < trace_cap) {
                trace_i[j * trace_cap + n_moves] = (int32_t)best_i;
                trace_r[j * trace_cap + n_moves] = best_r;
                trace_s[j * trace_cap + n_moves] = best_s;
            }
            q[best_i] = (uint8_t)best_r;
            const double *hrow = H + best_i * d_in;
            for (int64_t k = 0; k < d_in; ++k)
                g[k] += delta * hrow[k];
            ++n_moves;
        }
        moves[j] = n_moves;
        converged[j] = done;
    }
}

/* ---- one arg-min step on its own (Algorithm 1, the arg-min step), for
 * checking a score/arg-min kernel in isolation: returns per column the best
 * (i, r, s) or i = -1 when no move has a negative score. ---- */

void cdqo_argmin_f32(const float *Hdiag, const float *scale, const uint8_t *Q, const float *G,
                     int64_t d_out, int64_t d_in, int bits, int64_t group,
                     int32_t *out_i, int32_t *out_r, float *out_s)
{
    const int levels = 1 << bits;
    const int64_t n_grp = d_in / group;
    for (int64_t j = 0; j < d_out; ++j) {
        float best_s = 0.0f;
        int32_t best_i = -1, best_r = -1;
        for (int64_t i = 0; i < d_in; ++i) {
            const float ai = scale[j * n_grp + i / group];
            const int qi = Q[j * d_in + i];
            const float two_g = 2.0f * G[j * d_in + i];
            for (int r = 0; r < levels; ++r) {
                if (r == qi) continue;
                const float delta = ai * (float)(r - qi);
                const float s = delta * fmaf(delta, Hdiag[i], two_g);
                if (s < best_s) { best_s = s; best_i = (int32_t)i; best_r = r; }
            }
        }
        out_i[j] = best_i; out_r[j] = best_r; out_s[j] = best_s;
    }
}

/* ---- OWC-CD: greedy coordinate descent over per-group clipping strengths (Algorithm 3) ----
 *
 * Sub-channel grids (Section 3.2, "Initialization"): every group i of `group` consecutive
 * coordinates has its own clipping strength gamma_i on the grid {k/n_gamma : k = 1..n_gamma};
 * Eq. (2) per group gives its scale, bias and codes, hence its residual block
 * e^(i)(gamma) = a q + b - w  (the paper's Delta(i, gamma) with the opposite sign).
 * Per iteration, over all groups i and grid points beta, with d = e^(i)(beta) - e^(i)(gamma_i):
 *     score(i, beta) = d^T H_ii d + v_i^T d,   v = 2 H e,
 * is the exact change of the loss of Eq. (1); the smallest score is taken if it is negative,
 * then v <- v + 2 H[:, group i] d and gamma_i <- beta.
 *
 * Readings: the algorithm box initialises v with a leading minus sign, which contradicts both
 * its own update line and the requirement that the score be the loss change; v = +2He is used.
 * "Initialize clipping strengths" is not specified: every group starts at gamma = 1 (MinMax).
 * Ties: smallest score, then smallest group, then smallest grid index.
 *
 * Arithmetic: Eq. (2) and the residual in fp32 exactly as in the round-to-nearest routines
 * (a = (gamma*(hi-lo))/(2^c-1), q = clamp(rint((w-lo)/a)), e = fmaf(a,q,lo) - w); every sum
 * (v, scores) in fp64, so that another implementation that sums in a different order agrees
 * except at differences of order 1e-16.
 *
 * gamma_idx [d_out][n_grp] holds k (1..n_gamma) on exit.  trace arrays as in greedy CD
 * (trace_r holds the chosen grid index k).
 */
static void owc_group_residual(const float *w, int64_t group, int bits, float lo, float hi, int k, int n_gamma,
                               float *e_out, float *a_out, uint8_t *q_out)
{
    const float top = (float)((1 << bits) - 1);
    const float gamma = (float)k / (float)n_gamma;
    float a = (gamma * (hi - lo)) / top;
    if (!(a > 0.0f) || isinf(a)) a = 1.0f;
    for (int64_t m = 0; m < group; ++m) {
        float r = rintf((w[m] - lo) / a);
        if (r < 0.0f) r = 0.0f;
        if (r > top) r = top;
        if (e_out) e_out[m] = fmaf(a, r, lo) - w[m];
        if (q_out) q_out[m] = (uint8_t)r;
    }
    if (a_out) *a_out = a;
}

void cdqo_owc_cd(const float *H, const float *Wt, int64_t d_out, int64_t d_in, int bits, int64_t group,
                 int n_gamma, int64_t T, float *scale, float *zero, uint8_t *Q, int32_t *gamma_idx,
                 int32_t *moves, int32_t *converged,
                 int32_t *trace_i, int32_t *trace_r, double *trace_s, int64_t trace_cap)
{
    const int64_t n_grp = d_in / group;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t j = 0; j < d_out; ++j) {
        const float *w = Wt + j * d_in;
        float *tab = (float *)malloc(sizeof(float) * (size_t)n_gamma * d_in);   /* e(beta) for every beta */
        float *lo = (float *)malloc(sizeof(float) * n_grp), *hi = (float *)malloc(sizeof(float) * n_grp);
        float *e = (float *)malloc(sizeof(float) * d_in);
        double *v = (double *)malloc(sizeof(double) * d_in);
        double *d = (double *)malloc(sizeof(double) * group);
        int32_t *cur = gamma_idx + j * n_grp;
        for (int64_t i = 0; i < n_grp; ++i) {
            float l = w[i * group], h = w[i * group];
            for (int64_t m = 1; m < group; ++m) {
                if (w[i * group + m] < l) l = w[i * group + m];
                if (w[i * group + m] > h) h = w[i * group + m];
            }
            lo[i] = l; hi[i] = h;
            for (int k = 1; k <= n_gamma; ++k)
                owc_group_residual(w + i * group, group, bits, l, h, k, n_gamma,
                                   tab + (size_t)(k - 1) * d_in + i * group, NULL, NULL);
            cur[i] = n_gamma;                                   /* gamma = 1 */
        }
        for (int64_t m = 0; m < d_in; ++m) e[m] = tab[(size_t)(n_gamma - 1) * d_in + m];
        for (int64_t r = 0; r < d_in; ++r) {                    /* v = 2 H e */
            double acc = 0.0;
            for (int64_t m = 0; m < d_in; ++m) acc += (double)H[r * d_in + m] * (double)e[m];
            v[r] = 2.0 * acc;
        }
        int32_t n_moves = 0, done = 0;
        for (int64_t t = 0; t < T; ++t) {
            double best_s = 0.0;
            int64_t best_i = -1;
            int best_k = -1;
            for (int64_t i = 0; i < n_grp; ++i)
                for (int k = 1; k <= n_gamma; ++k) {
                    if (k == cur[i]) continue;
                    const float *en = tab + (size_t)(k - 1) * d_in + i * group;
                    for (int64_t m = 0; m < group; ++m) d[m] = (double)en[m] - (double)e[i * group + m];
                    double s = 0.0;
                    for (int64_t m = 0; m < group; ++m) {
                        double row = 0.0;
                        const float *hrow = H + (i * group + m) * d_in + i * group;
                        for (int64_t m2 = 0; m2 < group; ++m2) row += (double)hrow[m2] * d[m2];
                        s += d[m] * (row + v[i * group + m]);
                    }
                    if (s < best_s) { best_s = s; best_i = i; best_k = k; }
                }
            if (best_i < 0) { done = 1; break; }
            const float *en = tab + (size_t)(best_k - 1) * d_in + best_i * group;
            for (int64_t m = 0; m < group; ++m) d[m] = (double)en[m] - (double)e[best_i * group + m];
            for (int64_t r = 0; r < d_in; ++r) {                /* v += 2 H[:, group] d */
                double acc = 0.0;
                const float *hrow = H + r * d_in + best_i * group;
                for (int64_t m = 0; m < group; ++m) acc += (double)hrow[m] * d[m];
                v[r] += 2.0 * acc;
            }
            for (int64_t m = 0; m < group; ++m) e[best_i * group + m] = en[m];
            if (n_moves < trace_cap) {
                trace_i[j * trace_cap + n_moves] = (int32_t)best_i;
                trace_r[j * trace_cap + n_moves] = best_k;
                trace_s[j * trace_cap + n_moves] = best_s;
            }
            cur[best_i] = best_k;
            ++n_moves;
        }
        for (int64_t i = 0; i < n_grp; ++i) {
            float a;
            owc_group_residual(w + i * group, group, bits, lo[i], hi[i], cur[i], n_gamma, NULL, &a,
                               Q + j * d_in + i * group);
            scale[j * n_grp + i] = a;
            zero[j * n_grp + i] = lo[i];
        }
        moves[j] = n_moves;
        converged[j] = done;
        free(tab); free(lo); free(hi); free(e); free(v); free(d);
    }
}

/* ---- block coordinate descent with random blocks (Algorithm 2; Algorithm 5 for groups) ----
 *
 * Weight-space form, canonical fp32 arithmetic as in greedy CD.  The random partitions are an
 * input: parts[t*d_in + k*b + m] is member m of block b in iteration t (each row of parts is a
 * permutation of 0..d_in-1).  Per iteration every block b and every level tuple
 * r in {0..2^bits-1}^k is scored, tuples enumerated with the first member's level outermost:
 *     delta_m = a_m (r_m - q_m),          s_m = delta_m * fmaf(delta_m, H_mm, 2 g_m)
 *     s = s_0 + s_1 + ... (left to right), then for each pair m < m' in lexicographic order
 *     s = fmaf(delta_m * delta_m', 2 H_mm', s)
 * which is the loss change of moving the whole block.  The first strict minimum (block order,
 * then tuple order) is committed if it is negative: g <- g + delta_m H[member m, :] for
 * m = 0..k-1 in turn, codes of the block replaced.  An iteration without a negative score
 * changes nothing, but later partitions may still find moves, so all T iterations run.
 * k = 1 with the identity partition is greedy CD.
 *
 * trace_b = block index, trace_r = levels packed 4 bits per member (member 0 lowest), needs k <= 8.
 */
#define CDQO_MAX_K 8

void cdqo_bcd_f32(const float *H, const float *scale, uint8_t *Q, float *G, const int32_t *parts,
                  int64_t d_out, int64_t d_in, int bits, int64_t group, int k, int64_t T,
                  int32_t *moves, int32_t *trace_t, int32_t *trace_b, int32_t *trace_r, float *trace_s,
                  int64_t trace_cap)
{
    const int L = 1 << bits;
    const int64_t n_grp = d_in / group, n_blk = d_in / k;
    int64_t n_tuples = 1;
    for (int m = 0; m < k; ++m) n_tuples *= L;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t j = 0; j < d_out; ++j) {
        const float *a = scale + j * n_grp;
        uint8_t *q = Q + j * d_in;
        float *g = G + j * d_in;
        int32_t n_moves = 0;
        for (int64_t t = 0; t < T; ++t) {
            const int32_t *part = parts + t * d_in;
            float best_s = 0.0f;
            int64_t best_b = -1, best_tuple = -1;
            for (int64_t b = 0; b < n_blk; ++b) {
                const int32_t *mem = part + b * k;
                for (int64_t tup = 0; tup < n_tuples; ++tup) {
                    float delta[CDQO_MAX_K];
                    int64_t rest = tup;
                    for (int m = k - 1; m >= 0; --m) {           /* member 0 is the most significant digit */
                        const int r = (int)(rest % L);
                        rest /= L;
                        delta[m] = a[mem[m] / group] * (float)(r - (int)q[mem[m]]);
                    }
                    float s = 0.0f;
                    for (int m = 0; m < k; ++m) {
                        const int64_t c = mem[m];
                        const float sm = delta[m] * fmaf(delta[m], H[c * d_in + c], 2.0f * g[c]);
                        s = (m == 0) ? sm : s + sm;
                    }
                    for (int m = 0; m < k; ++m)
                        for (int m2 = m + 1; m2 < k; ++m2)
                            s = fmaf(delta[m] * delta[m2], 2.0f * H[(int64_t)mem[m] * d_in + mem[m2]], s);
                    if (s < best_s) { best_s = s; best_b = b; best_tuple = tup; }
                }
            }
            if (best_b < 0) continue;
            const int32_t *mem = part + best_b * k;
            int64_t rest = best_tuple;
            int r_new[CDQO_MAX_K];
            for (int m = k - 1; m >= 0; --m) { r_new[m] = (int)(rest % L); rest /= L; }
            int32_t packed = 0;
            for (int m = 0; m < k; ++m) {
                const int64_t c = mem[m];
                const float delta = a[c / group] * (float)(r_new[m] - (int)q[c]);
                const float *hrow = H + c * d_in;
                for (int64_t x = 0; x < d_in; ++x) g[x] = fmaf(delta, hrow[x], g[x]);
                q[c] = (uint8_t)r_new[m];
                packed |= r_new[m] << (4 * m);
            }
            if (n_moves < trace_cap) {
                trace_t[j * trace_cap + n_moves] = (int32_t)t;
                trace_b[j * trace_cap + n_moves] = (int32_t)best_b;
                trace_r[j * trace_cap + n_moves] = packed;
                trace_s[j * trace_cap + n_moves] = best_s;
            }
            ++n_moves;
        }
        moves[j] = n_moves;
    }
}

/* ---- cyclic coordinate descent (the fixed-order variant the paper contrasts greedy CD with:
 * Section 1 and the appendix comparison with QuantEase) ----
 *
 * Same single-coordinate move and the same canonical fp32 arithmetic as greedy CD, but the
 * coordinate is not chosen by an arg-min over all of them: visit t looks at coordinate
 * i = t mod d_in only, scores every level r (delta = a (r - q_i), s = delta * fmaf(delta, H_ii, 2 g_i)),
 * and commits the first strict minimum if it is negative (g <- g + delta H[i, :]).  T counts visits
 * (d_in visits = one epoch).  The column stops early once d_in consecutive visits made no move:
 * it is then at a coordinate-wise optimum.  iters[j] = visits performed.
 */
void cdqo_cyclic_cd_f32(const float *H, const float *scale, uint8_t *Q, float *G,
                        int64_t d_out, int64_t d_in, int bits, int64_t group, int64_t T,
                        int32_t *moves, int32_t *iters, int32_t *converged,
                        int32_t *trace_i, int32_t *trace_r, float *trace_s, int64_t trace_cap)
{
    const int L = 1 << bits;
    const int64_t n_grp = d_in / group;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t j = 0; j < d_out; ++j) {
        const float *a = scale + j * n_grp;
        uint8_t *q = Q + j * d_in;
        float *g = G + j * d_in;
        int32_t n_moves = 0, done = 0;
        int64_t idle = 0, t = 0;
        for (; t < T; ++t) {
            if (idle == d_in) { done = 1; break; }
            const int64_t i = t % d_in;
            const float ai = a[i / group], hii = H[i * d_in + i], two_g = 2.0f * g[i];
            float best_s = 0.0f;
            int best_r = -1;
            for (int r = 0; r < L; ++r) {
                const float delta = ai * (float)(r - (int)q[i]);
                const float s = delta * fmaf(delta, hii, two_g);
                if (s < best_s) { best_s = s; best_r = r; }
            }
            if (best_r < 0) { ++idle; continue; }
            idle = 0;
            const float delta = ai * (float)(best_r - (int)q[i]);
            const float *hrow = H + i * d_in;
            for (int64_t k = 0; k < d_in; ++k) g[k] = fmaf(delta, hrow[k], g[k]);
            q[i] = (uint8_t)best_r;
            if (n_moves < trace_cap) {
                trace_i[j * trace_cap + n_moves] = (int32_t)i;
                trace_r[j * trace_cap + n_moves] = best_r;
                trace_s[j * trace_cap + n_moves] = best_s;
            }
            ++n_moves;
        }
        if (!done && idle == d_in) done = 1;
        moves[j] = n_moves;
        iters[j] = (int32_t)t;
        converged[j] = done;
    }
}
