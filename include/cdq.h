/*
 * libcdq -- the hot path of CDQuant (arXiv 2406.17542, "Greedy Coordinate Descent for Accurate
 * LLM Quantization") for AMD MI355X (gfx950).  C ABI: plain pointers and sizes only.
 *
 * Problem (paper Section 3, Notation and Eq. (1)): a linear layer with weight W [d_in x d_out]
 * and calibration inputs X [n x d_in] is quantized column by column; every output column w is
 * replaced by a*q + b with integer codes q in {0..2^c-1}, so as to minimise
 * ||X (w - a q - b)||^2 = e^T H e,  H = X^T X,  e = a q + b - w.
 * With sub-channel quantization (Section 3.2) a and b are constant on groups of `group`
 * consecutive input coordinates.
 *
 * Conventions common to every call
 *   - Every data pointer is a DEVICE pointer owned by the caller; the library never frees or
 *     keeps one.  `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work on that stream and return; they do not synchronise the device.
 *   - Wt, Q are [d_out][d_in] row-major: row j is output column j of the paper's W (the layout
 *     of a torch nn.Linear weight).  scale, zero are [d_out][d_in/group] (the paper's a, b).
 *     H is [d_in][d_in] fp32, full storage, and must be symmetric.
 *   - bits in {2,3,4}; d_in % group == 0; group == d_in means per-channel.
 *   - `workspace` is device scratch of at least cdq_workspace_bytes(op, ...) bytes, 256-byte
 *     aligned; its contents are undefined afterwards.  Calls sharing a workspace must be
 *     ordered on one stream.
 *   - Return value: CDQ_OK or a negative error code; nothing is enqueued when an argument
 *     check fails.  No global mutable state.
 */
#ifndef CDQ_H
#define CDQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CDQ_OK            0
#define CDQ_EINVAL       (-1)   /* null pointer, bad shape, bits not in {2,3,4}, d_in % group != 0 ... */
#define CDQ_EWORKSPACE   (-2)   /* workspace missing, misaligned or too small */
#define CDQ_EHIP         (-3)   /* a HIP runtime call failed (launch error, wrong device ...) */
#define CDQ_EUNSUPPORTED (-4)   /* valid request outside what the kernels cover (e.g. d_in too large) */

#define CDQ_F32  0
#define CDQ_BF16 1

/* operations for cdq_workspace_bytes */
#define CDQ_OP_HESSIAN   0
#define CDQ_OP_GREEDY_CD 1
#define CDQ_OP_LOSS      2
#define CDQ_OP_INIT_OWC  3
#define CDQ_OP_INIT_OWC_CD 4
#define CDQ_OP_BCD       5   /* n = T, the number of iterations */
#define CDQ_OP_CYCLIC_CD 6

#define CDQ_MAX_D_IN 36864      /* largest d_in the register-resident CD kernel covers (above 32768 only
                                   with d_in and group multiples of 4 and 16-byte aligned H) */

/* Per-column outcome of cdq_greedy_cd. */
typedef struct {
    int32_t moves;        /* committed coordinate updates */
    int32_t iters;        /* iterations executed (== moves, +1 if the last one found no move) */
    int32_t converged;    /* 1: stopped because no single-coordinate move lowers the loss */
    float   last_score;   /* score (loss change) of the last committed move, 0 if none */
} cdq_col_stats;

/* Optional controls for cdq_greedy_cd_ex; zero-initialise for defaults. */
typedef struct {
    int32_t  waves_per_column;  /* 0 = choose; else 1,2,4,8,16 wavefronts cooperating on a column */
    int32_t  elems_per_lane;    /* 0 = choose; else 4,8,16,32 coordinates held per lane; 24 or 36, and 32 for
                                   16-byte aligned layers, with 16 wavefronts are the kernel that keeps the
                                   Hessian diagonal in LDS, the one chosen for d_in above 16384 */
    int32_t  exact_scorer_only; /* 1 = two-level scorer on every iteration: per coordinate the two levels next to the
                                   parabola's minimiser, both by the formula below -- the arg-min of Algorithm 1 over
                                   all levels, unconditionally (1.15 to 1.3 times the loop time).
                                   0 (default) = nearest-level scorer: one level per coordinate; the iteration is
                                   redone with the two-level scorer when the winner's minimiser lies within 2^-9 of a
                                   half-integer or no move was found.  A coordinate whose minimiser is farther than
                                   that from a half-integer is scored identically by both.  The selected move can
                                   differ from Algorithm 1's arg-min in one situation only: a coordinate OTHER than
                                   the winner whose minimiser lies within 2^-15 of a half-integer gets the worse of
                                   its two levels -- worse by at most 2^-15 a^2 H_ii + 2^-21 |s| -- and its better
                                   level would have beaten the winner by less than that.  Both moves then lower the
                                   loss, by amounts that agree to about 1e-5 of a grid step's worth. */
    int32_t  teams_per_cu;      /* 0 = choose; 1 = one column per compute unit at a time with its state in registers;
                                   2 = two, with the Hessian diagonal in LDS and 64 registers per lane, so that one
                                   column is scored while the other waits for its row of H.  2 exists for 16 wavefronts
                                   x 16 coordinates per lane (8192 < d_in <= 16384, 16-byte chunks) only, CDQ_EINVAL
                                   elsewhere; chosen there when the layer has more columns than the chip has compute
                                   units.  Same moves either way. */
    int32_t *trace;             /* NULL, or [d_out][trace_cap]: move m of column j is stored as
                                   i* * 64 + (u* + 32), u* = r* - q_i* the signed level change */
    int64_t  trace_cap;
    float   *G_out;             /* NULL, or [d_out][d_in]: g = H e as maintained at exit */
    void    *ev_loop_begin;     /* NULL, or hipEvent_t recorded on `stream` just before ... */
    void    *ev_loop_end;       /* ... and just after the iteration-loop kernel, so a caller can
                                   time the loop apart from the gradient initialisation */
    float   *G0;                /* NULL, or [d_out][d_in], 16-byte aligned: the start gradient H e of the codes passed in, as
                                   cdq_gradient or cdq_init_owc's G_out give it.  The gradient initialisation is then
                                   skipped, the workspace only needs 4 d_in bytes (rounded up to 256), and the array is
                                   OVERWRITTEN (the loop uses it as scratch).  A G0 that is not the gradient of
                                   (scale, zero, Q) makes the result meaningless; nothing checks it. */
} cdq_cd_options;

const char *cdq_strerror(int code);

/* Bytes of workspace an operation needs for the given shape (host-only, no GPU access).
 * n is used by CDQ_OP_HESSIAN only. */
size_t cdq_workspace_bytes(int op, int64_t n, int64_t d_out, int64_t d_in);

/*
 * Hessian of the layer objective: H = X^T X (paper Section 3, Notation; Algorithm 1,
 * "Compute Hessian"), optionally damped H += lambda*I as in Section 4 ("we regularize the
 * Hessian ... by adding lambda I").  The paper does not give lambda; here
 * lambda = lambda_rel * mean(diag H), lambda_rel = 0 disables it.
 *   X           [n][d_in] row-major, bf16 (CDQ_BF16) or fp32 (CDQ_F32); d_in % 8 == 0 for bf16,
 *               % 4 == 0 for fp32 (rows must be 16-byte aligned)
 *   H           [d_in][d_in] fp32 out (both triangles written, exactly symmetric)
 *   accumulate  0: H = X^T X;  1: H += X^T X (streaming over chunks of tokens; H must already
 *               hold a symmetric matrix).
 *   lambda_rel  damping added at the end of THIS call, after the sum, from the diagonal H then has.
 *               When streaming, pass it on the last chunk only and 0 on the others: a non-zero
 *               value on every chunk would add damping once per call.
 * Products are exact (bf16) or fp32, accumulation is fp32 on the matrix cores; the summation
 * order over tokens is fixed, so results are reproducible run to run.
 */
int cdq_hessian(const void *X, int x_dtype, int64_t n, int64_t d_in, float *H, int accumulate,
                float lambda_rel, void *workspace, size_t workspace_bytes, void *stream);

/*
 * MinMax grid and round-to-nearest codes: Eq. (2) with clipping strength gamma = 1, per
 * (column, group): zero = min w, scale = (max w - min w)/(2^bits - 1),
 * Q = clamp(round_half_even((w - zero)/scale), 0, 2^bits - 1), all in IEEE fp32.
 * A constant group gets scale = 1 and codes 0.
 *   Wt [d_out][d_in] in;  scale, zero [d_out][d_in/group] out;  Q [d_out][d_in] out.
 */
int cdq_init_rtn(const float *Wt, int64_t d_out, int64_t d_in, int bits, int64_t group,
                 float *scale, float *zero, uint8_t *Q, void *stream);

/*
 * Optimal Weight Clipping, the paper's initialisation for per-channel CD (Section 3.1,
 * "Initializing a, b, q"; Section 4: grid size 50): Eq. (2) with the clipping strength gamma
 * chosen per column by grid search on the layer loss of Eq. (1):
 *   zero = min w, scale = gamma (max w - min w)/(2^bits - 1), Q = clamp(round((w-zero)/scale)),
 *   gamma = argmin over {k/n_gamma : k = 1..n_gamma} of e^T H e (fp64); equal losses keep the
 *   larger gamma.  Only the upper end is clipped, as Eq. (2) is written.
 * Needs group == d_in (one clipping strength per column), else CDQ_EUNSUPPORTED.
 *   scale, zero [d_out] out; Q [d_out][d_in] out; gamma_out NULL or [d_out] fp32;
 *   loss_out NULL or [d_out] fp64 (loss of the chosen grid point);
 *   researched NULL or one int32 (device): number of columns that failed the check below (not written when d_out == 0).
 *   G_out NULL or [d_out][d_in] fp32: the gradient H e of the returned grid and codes, bit for bit what cdq_gradient
 *   computes for them, for cdq_cd_options.G0.  It costs less here than there: the fp64 pass over every column's best
 *   grid point is run as the full product E H, which leaves the gradient and yields the loss from the same sums; only
 *   the columns that end at another grid point are multiplied again.
 * Cost and safeguard.  The exhaustive search costs n_gamma passes of the fp64 loss kernel (d_out d_in^2 FLOP each).  When
 * d_in is a multiple of 128 (at least 256) and 4 <= n_gamma <= 255, every grid point is first evaluated in fp16 on the
 * matrix cores in the normalised form s^2 f^T R f (R = H scaled to unit diagonal, f = e sqrt(diag H) / s), and only the
 * grid points within `screen_margin` (relative; 0 selects the default 3e-3) of a column's smallest such value -- one or
 * two per column on typical layers -- are evaluated in fp64, which decides among them as above.  The fp16 value is an
 * estimate (its relative error stayed below 3e-4 on the test layers, but it grows when channels are nearly collinear, where
 * rounding R moves f^T R f), so it is checked column by column: the chosen grid point has both values, and a column where
 * they differ by more than a third of the margin is searched exhaustively in fp64 after all.  The result therefore equals
 * the exhaustive search's for every column that fails the check, and for the others whenever the fp16 error at the
 * grid points that were not evaluated is no larger than the margin -- three times what was measured on that column.
 * H needs a positive diagonal for the fp16 stage to say anything (otherwise every grid point fails over to fp64).
 * H is taken to be symmetric and only its blocks on and above the diagonal are multiplied, see cdq_loss.
 */
int cdq_init_owc(const float *H, const float *Wt, int64_t d_out, int64_t d_in, int bits, int64_t group,
                 int n_gamma, float screen_margin, float *scale, float *zero, uint8_t *Q, float *gamma_out,
                 double *loss_out, int32_t *researched, float *G_out, void *workspace, size_t workspace_bytes,
                 void *stream);

/*
 * OWC-CD, the paper's initialisation for sub-channel grids (Algorithm 3; Section 3.2,
 * "Initialization"): greedy coordinate descent over one clipping strength per group, on the grid
 * {k/n_gamma : k = 1..n_gamma}, every group starting at 1 (MinMax).  Per iteration the move
 * (group i, grid point k) with the smallest exact loss change d^T H_ii d + 2 (H e)_i^T d,
 * d = e_i(k) - e_i(current), is taken if negative (ties: smallest group, then smallest k);
 * T iterations at most (the paper uses T = d_in/group).  All sums in fp64.
 *   scale, zero [d_out][d_in/group] out; Q [d_out][d_in] out (Eq. (2) with the chosen strengths);
 *   gamma_idx NULL or [d_out][d_in/group] int32 (chosen k); moves NULL or [d_out] int32;
 *   trace NULL or [d_out][trace_cap] int32: move m is stored as group*4096 + k.
 *   variant 0: tiled kernel (needs group % 4 == 0 and 16-byte aligned H, Wt; otherwise the
 *              simple kernel is taken); MinMax start and its gradient come from the RTN and
 *              fp64 GEMM kernels, which needs a workspace of CDQ_OP_INIT_OWC_CD size.
 *   variant 1: simple kernel (one pass per quantity, no workspace); same results up to fp64
 *              rounding of the scores.
 * The column's state is kept in LDS: roughly max(8*d_in + 8*n_gamma*d_in/group, 4*n_gamma*group)
 * + 8*d_in + 16*n_gamma*d_in/group bytes <= 160 KiB, else CDQ_EUNSUPPORTED.
 */
int cdq_init_owc_cd(const float *H, const float *Wt, int64_t d_out, int64_t d_in, int bits, int64_t group,
                    int n_gamma, int64_t T, float *scale, float *zero, uint8_t *Q, int32_t *gamma_idx,
                    int32_t *moves, int32_t *trace, int64_t trace_cap, int variant, void *workspace,
                    size_t workspace_bytes, void *stream);

/*
 * Block coordinate descent with random blocks (Algorithm 2; Algorithm 5 for groups), block size
 * k = 2 (CDQ_EUNSUPPORTED otherwise; k = 1 is cdq_greedy_cd), weight-space form, canonical fp32
 * arithmetic.  The random partitions are an input so that every implementation sees the same
 * ones:  parts [T][d_in] int32, device; row t is a permutation of 0..d_in-1 and block b of
 * iteration t is (parts[t][2b], parts[t][2b+1]); all columns use the same partitions.  Rows that
 * are not permutations are detected on the device: then nothing is changed and moves[j] = -1.
 * Per iteration the block and level pair with the smallest loss change
 *     s = fma(di*dk, 2 H_ik, di*fma(di, H_ii, 2 g_i) + dk*fma(dk, H_kk, 2 g_k)),  d = a (r - q),
 * over all d_in/2 blocks and 4^bits level pairs is committed if negative (ties: first block of
 * the partition, then smaller r_i, then smaller r_k): g += di H[i,:], then g += dk H[k,:].
 * All T iterations run (a later partition may find moves an earlier one did not).
 *   Q [d_out][d_in] in/out; moves NULL or [d_out] int32 out; G_out NULL or [d_out][d_in] fp32:
 *   g = He of the final codes as maintained by the updates;
 *   trace NULL or [d_out][trace_cap][4] int32: iteration, block, r_i | r_k<<4, score bits.
 *   flags bit 0 clear: pairs that provably hold no improving move are not scored (with
 *   u = |2 g| / (H_ii a), or 0 for a code at the end of its grid that g points past, and
 *   rho = |H_ik| / sqrt(H_ii H_kk): (1 - u_i - 2^-14)(1 - u_k - 2^-14) >= rho^2, both factors >= 0);
 *   set: every pair is scored.
 *   flags bit 1 set: one column per workgroup also where the kernel that gives a workgroup
 *   several columns applies (d_in % 8 == 0 and the columns' state fits LDS).
 *   flags bit 2 set: the wide-layer kernel with 8 columns per workgroup whatever the shape.  Same
 *   results for every value of flags;
 *   the bits exist for tests and timing.
 * d_in even, at most 65534.  Three kernels give the same results: several columns per workgroup
 * with their state in LDS (d_in % 16 == 0, d_in up to about 4700), one column per workgroup with
 * its state in LDS (d_in <= 8192, d_in % 4 == 0, 16-byte aligned H), and for wider or differently
 * aligned layers up to 16 columns per workgroup with only the pair test's 16-bit margins in LDS
 * and everything else in global memory.  Workspace of CDQ_OP_BCD size (n = T):
 * d_out*d_in*8 + T*(d_in/2)*12 bytes and change.
 */
int cdq_bcd(const float *H, const float *Wt, const float *scale, const float *zero, uint8_t *Q,
            int64_t d_out, int64_t d_in, int bits, int64_t group, int k, const int32_t *parts, int64_t T,
            int32_t *moves, float *G_out, int32_t *trace, int64_t trace_cap, int flags,
            void *workspace, size_t workspace_bytes, void *stream);

/*
 * Cyclic (fixed-order) coordinate descent: the variant without an arg-min over coordinates that the
 * paper contrasts greedy CD with (Section 1; appendix comparison with QuantEase).  Visit t handles
 * coordinate t mod d_in: all levels are scored with the single-coordinate score of Algorithm 1,
 * s = delta*fma(delta, H_ii, 2 g_i), delta = a (r - q_i), and the first strict minimum is
 * committed if negative.  T counts visits (one epoch = d_in visits); a column stops once d_in
 * consecutive visits made no move (stats.converged = 1); stats.iters = visits performed.
 *   Q in/out; stats NULL or [d_out]; G_out NULL or [d_out][d_in]; trace NULL or
 *   [d_out][trace_cap] int32: move m is stored as (i << 7) | r.
 * Needs d_in % 4 == 0, 16-byte aligned H, 9*d_in bytes of LDS; workspace of CDQ_OP_CYCLIC_CD size.
 */
int cdq_cyclic_cd(const float *H, const float *Wt, const float *scale, const float *zero, uint8_t *Q,
                  int64_t d_out, int64_t d_in, int bits, int64_t group, int64_t T,
                  cdq_col_stats *stats, float *G_out, int32_t *trace, int64_t trace_cap,
                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * Gradient initialisation of Algorithm 1 ("Compute gradient g at q0"), in weight space:
 * G[j][:] = H e_j with e_j = scale*Q[j] + zero - Wt[j] (the paper's g is (2/a) times this).
 * fp32 inputs, fp64 accumulation on the matrix cores, one rounding to fp32.
 *   G [d_out][d_in] out.
 */
int cdq_gradient(const float *H, const float *Wt, const float *scale, const float *zero,
                 const uint8_t *Q, int64_t d_out, int64_t d_in, int64_t group, float *G,
                 void *stream);

/*
 * Greedy coordinate descent, Algorithm 1 (Algorithm 4 of the appendix when group < d_in),
 * run independently for all d_out columns.  Per column, up to T times: over all coordinates i
 * and levels r != q_i take the move with the smallest
 *     s(i,r) = delta * fma(delta, H_ii, 2 g_i),  delta = scale_grp(i) * (r - q_i)
 * (the exact loss change; the paper's score times scale^2); ties go to the smallest i, then
 * the smallest r.  If s >= 0 the column is at a coordinate-wise optimum and stops.  Otherwise
 * commit Q[j][i*] = r* and g <- fma(delta*, H[i*][:], g).  All T iterations run inside one
 * kernel launch with g held in registers.
 *   Q      in: initial codes q0 (from cdq_init_rtn, cdq_init_owc, or a previous run);
 *          out: final codes.
 *   stats  NULL or [d_out] out.
 *   T      >= 0 (0 leaves Q unchanged).
 * Needs d_in <= CDQ_MAX_D_IN, else CDQ_EUNSUPPORTED.
 */
int cdq_greedy_cd(const float *H, const float *Wt, const float *scale, const float *zero,
                  uint8_t *Q, int64_t d_out, int64_t d_in, int bits, int64_t group, int64_t T,
                  cdq_col_stats *stats, void *workspace, size_t workspace_bytes, void *stream);

/* Same, with explicit launch shape and optional move trace / final gradient (opts may be NULL). */
int cdq_greedy_cd_ex(const float *H, const float *Wt, const float *scale, const float *zero,
                     uint8_t *Q, int64_t d_out, int64_t d_in, int bits, int64_t group, int64_t T,
                     cdq_col_stats *stats, const cdq_cd_options *opts,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * The launch shape cdq_greedy_cd takes for a layer when nothing is forced: wavefronts cooperating on
 * a column, coordinates held per lane (64 * waves * elems >= d_in) and, if teams_per_cu is not NULL,
 * columns resident per compute unit (cdq_cd_options.teams_per_cu).  Host-only, no GPU access.
 * `aligned16` tells whether H rows and Q rows are 16- and 4-byte aligned (they are when the base
 * pointers are and d_in % 4 == 0); without it the kernels fall back to scalar loads.
 * Returns CDQ_EUNSUPPORTED where cdq_greedy_cd would.
 */
int cdq_greedy_cd_shape(int64_t d_out, int64_t d_in, int64_t group, int aligned16,
                        int32_t *waves_per_column, int32_t *elems_per_lane, int32_t *teams_per_cu);

/*
 * One iteration of Algorithm 1 as separate steps, on a gradient G = E H kept in global memory
 * (from cdq_gradient).  Any d_in; one launch each.
 *   cdq_score_argmin   the arg-min step: per column the move (i, r) with the smallest score
 *                      s = delta*fma(delta, Hdiag_i, 2 G_ji), ties to the smallest i then r;
 *                      best_i = best_r = -1 and best_s = 0 when no move has s < 0.
 *                      Hdiag [d_in] is the diagonal of H.  best_i, best_r [d_out] int32, best_s [d_out].
 *   cdq_gather_update  the code- and gradient-update steps for those moves: Q[j][i] = r,
 *                      G[j][:] = fma(delta, H[i][:], G[j][:]); columns with best_i < 0 are left
 *                      alone.  moves: NULL or [d_out] int32 counters, incremented per committed move.
 *   cdq_greedy_cd_stepwise  gradient init + T such iteration pairs (2T launches, no host sync);
 *                      same results as cdq_greedy_cd; workspace of CDQ_OP_GREEDY_CD size.
 *                      `moves` (NULL or [d_out], zeroed by the caller) counts committed moves.
 */
int cdq_score_argmin(const float *Hdiag, const float *scale, const uint8_t *Q, const float *G,
                     int64_t d_out, int64_t d_in, int bits, int64_t group,
                     int32_t *best_i, int32_t *best_r, float *best_s, void *stream);
int cdq_gather_update(const float *H, const float *scale, uint8_t *Q, float *G, int64_t d_out,
                      int64_t d_in, int64_t group, const int32_t *best_i, const int32_t *best_r,
                      int32_t *moves, void *stream);
int cdq_greedy_cd_stepwise(const float *H, const float *Wt, const float *scale, const float *zero,
                           uint8_t *Q, int64_t d_out, int64_t d_in, int bits, int64_t group, int64_t T,
                           int32_t *moves, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Layer loss of Eq. (1) from the codes: loss_per_col[j] = e_j^T H e_j, loss_total = sum_j
 * (= ||X (W - W_hat)||_F^2).  fp32 inputs, fp64 accumulation, fixed summation order.
 * H is taken to be symmetric, as cdq_hessian writes it: only its 128 x 128 blocks on and above
 * the diagonal are read, those above counted twice.
 *   loss_per_col  NULL or [d_out] fp64 out;  loss_total  NULL or one fp64 out (device).
 */
int cdq_loss(const float *H, const float *Wt, const float *scale, const float *zero,
             const uint8_t *Q, int64_t d_out, int64_t d_in, int64_t group,
             double *loss_per_col, double *loss_total,
             void *workspace, size_t workspace_bytes, void *stream);

/*
 * cdq_loss for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same sums in
 * the same order and therefore the same results as cdq_loss; the partial sums go to an array that
 * is part of the library's device image (CDQ_LOSS_STATIC_SCRATCH_BYTES per GPU, held until the
 * process ends) instead of a workspace.  The call allocates and frees nothing.
 * Layers for which cdq_workspace_bytes(CDQ_OP_LOSS, 0, d_out, d_in) exceeds
 * CDQ_LOSS_STATIC_SCRATCH_BYTES are rejected with CDQ_EUNSUPPORTED before any GPU work (the limit
 * covers d_out * ceil(d_in/128) up to about 2.1 million, e.g. 32768 x 8192).
 * All calls on one GPU share that GPU's array: calls that overlap on one GPU (different streams,
 * different threads) race; order them on one stream.  Nothing has to be cleared between calls.
 */
#define CDQ_LOSS_STATIC_SCRATCH_BYTES (24u << 20)
int cdq_loss_static(const float *H, const float *Wt, const float *scale, const float *zero,
                    const uint8_t *Q, int64_t d_out, int64_t d_in, int64_t group,
                    double *loss_per_col, double *loss_total, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CDQ_H */
