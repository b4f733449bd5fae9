// Greedy coordinate descent (paper Algorithm 1; Algorithm 4 for sub-channel grids): all T
// iterations of one output column run inside one kernel, with the column's state -- twice the
// gradient g = H e, the codes q, the Hessian diagonal -- held in registers.  A column is owned
// by a team of W wavefronts (one workgroup); columns never interact, so there is no grid-wide
// synchronisation and no launch per iteration.
//
// Per iteration (Algorithm 1, the arg-min, gradient-update and code-update steps):
//   1. every lane scores its coordinates.  The score s(r) = delta*fma(delta, H_ii, 2 g_i),
//      delta = a*(r - q_i), is a convex parabola in r, so its minimum over the integer levels
//      sits next to the clamped continuous minimiser rf = q_i - 2g_i/(2 a H_ii).
//        fast scorer : scores only the level nearest to rf (about 12 VALU ops per coordinate).
//        exact scorer: scores floor(rf) and ceil(rf), both with exactly the formula above, so it
//                      selects what a scan of all 2^c levels would select (the levels left out
//                      are >= 0.75 a^2 H_ii worse, far above rounding error).
//      For one coordinate the two can only disagree when rf is within rounding distance of a
//      half-integer (within 2^-15: there the fp32 scores of the two neighbouring levels round to within
//      a few units of each other) or when no strictly improving move is left.  The fast scorer
//      therefore flags a winner whose rf lies within 2^-9 of a half-integer, and the iteration is
//      redone with the exact scorer when the winner is flagged or when no move was found.  What this
//      does not catch is a coordinate that is NOT the winner, sits within 2^-15 of a half-integer, was
//      given the worse of its two levels (worse by at most 2^-15 a^2 H_ii + 2^-21 |s|) and would have
//      won with the better one: the winner is then taken instead, a move whose gain agrees with the
//      arg-min's to about 1e-5 of a grid step's worth.  Checking every coordinate costs three to five
//      more vector instructions per coordinate in a loop that is bound by exactly those; callers that
//      need Algorithm 1's arg-min unconditionally set exact_scorer_only.
//   2. the team reduces (ordered score, then i, then level change) with unsigned minima: the
//      result does not depend on the reduction tree and implements the tie-break "smallest s,
//      then smallest i, then smallest r".  Within a wavefront: DPP minima over the 32-bit score
//      image, then the payload of the winning lane by readlane; across wavefronts: one 64-bit
//      slot per wavefront in LDS, double-buffered, one barrier.
//   3. the H row of the winning coordinate is streamed with coalesced 16-byte loads and folded
//      into the registers: 2g <- fma(2 delta, H[i*][:], 2g), which is bit-identical to updating g.
#include "cdq_internal.h"
#include "wave_min.h"

namespace cdq {

namespace {

constexpr float kHalfWindow = 1.0f / 512.0f;     // |frac(rf) - 1/2| below this: neighbouring levels may tie

// reciprocal of the parabola's curvature 2 a H_ii.  It only steers which levels are scored (every score is computed from
// H_ii itself), so the hardware's one-instruction reciprocal, good to one unit in the last place, serves: a level chosen
// differently because of that last place lies at a half-integer minimiser, where the two-level scorer takes over anyway.
// The kernels that keep the diagonal in LDS recompute it at every use; a correctly rounded division there cost more than
// the scoring itself (a dozen instructions and a branch per coordinate).
__device__ __forceinline__ float curvature_inv(float h, float a) {
    return (h > 0.0f) ? fminf(__builtin_amdgcn_rcpf(2.0f * a * h), 3.0e38f) : 0.0f;
}

// LDSH: the Hessian diagonal lives in LDS (each lane reads back only what it wrote, so no barrier is involved) and
// the curvature reciprocal is recomputed per use -- the same operations on the same values, hence the same numbers.
// It frees 2E registers per lane and is what lets a team of 16 wavefronts cover d_in up to 36864 (the diagonal of a
// longer column would not fit the 160 KiB of LDS).
// FF: recognise a column that moves one coordinate up and down for the rest of its budget and jump to the end (see the loop).
template <int W, int E, int VEC, bool LDSH, bool FF>
__device__ __forceinline__ void cd_fused_body(
    const float* __restrict__ H, const float* __restrict__ hdiag, float* G0,
    const float* __restrict__ scale, uint8_t* __restrict__ Q, int d_in, int bits, int group, int group_shift,
    int n_grp, int T, int exact_only, cdq_col_stats* __restrict__ stats, int32_t* __restrict__ trace,
    int64_t trace_cap, float* __restrict__ G_out) {
    constexpr int NCH = E / VEC;              // chunks of VEC consecutive coordinates per lane
    constexpr int STRIDE = 64 * W * VEC;      // coordinates covered by the team per chunk
    __shared__ unsigned long long slots[2][16];
    extern __shared__ __attribute__((aligned(16))) float hd_lds[];     // LDSH: [NCH][64 W][VEC]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int64_t j = blockIdx.x;
    const float* scale_j = scale + j * n_grp;
    uint8_t* Qj = Q + j * (int64_t)d_in;
    const float* G0j = G0 + j * (int64_t)d_in;    // the start gradient; once it is loaded, the row serves as a snapshot of 2g (below)
    const float top = (float)((1 << bits) - 1);

    float g2[E], hd[LDSH ? 1 : E], cinv[LDSH ? 1 : E], a_c[NCH];
    uint32_t qpack[NCH];

    // lanes past the end of the column load from its start and then zero what they loaded: no load sits in a divergent
    // branch, so all of them are in flight together
    float gl[E], hl[E];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int base = c * STRIDE + tid * VEC;
        const int b = base < d_in ? base : 0;
        const int gi = (n_grp == 1) ? 0 : (group_shift >= 0 ? (b >> group_shift) : (b / group));
        a_c[c] = scale_j[gi];
        if constexpr (VEC == 4) {
            qpack[c] = *reinterpret_cast<const uint32_t*>(Qj + b);
            const float4 g4 = *reinterpret_cast<const float4*>(G0j + b), h4 = *reinterpret_cast<const float4*>(hdiag + b);
            gl[c * 4 + 0] = g4.x; gl[c * 4 + 1] = g4.y; gl[c * 4 + 2] = g4.z; gl[c * 4 + 3] = g4.w;
            hl[c * 4 + 0] = h4.x; hl[c * 4 + 1] = h4.y; hl[c * 4 + 2] = h4.z; hl[c * 4 + 3] = h4.w;
        } else {
            qpack[c] = Qj[b];
            gl[c] = G0j[b];
            hl[c] = hdiag[b];
        }
    }
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const bool valid = c * STRIDE + tid * VEC < d_in;
        if (!valid) { a_c[c] = 1.0f; qpack[c] = 0; }
        const float a = a_c[c];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            const int e = c * VEC + v;
            const float g = valid ? gl[e] : 0.0f, h = valid ? hl[e] : 0.0f;
            g2[e] = 2.0f * g;
            if constexpr (LDSH) {
                hd_lds[(c * 64 * W + tid) * VEC + v] = h;
            } else {
                hd[e] = h;
                cinv[e] = curvature_inv(h, a);
            }
        }
    }
    // The lane's index as the loop sees it.  In the kernels with the diagonal in LDS it is passed through an empty asm at
    // the top of every iteration, so that what is derived from it (chunk offsets, validity masks, LDS addresses: two dozen
    // values that never change) is recomputed where it is used, one or two instructions each, instead of being hoisted out
    // of the loop into registers that do not exist and reloaded from scratch memory in front of every row load.
    int tl = tid;
    // Hessian diagonal and curvature reciprocal of the lane's chunk c
    auto diag_of = [&](int c, float (&h)[VEC], float (&ci)[VEC]) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            if constexpr (LDSH) {
                h[v] = hd_lds[(c * 64 * W + tl) * VEC + v];
                // curvature_inv without its guards: they only matter for H_ii = 0 (a dead channel: its row of H and so its
                // gradient are zero) and for a curvature that underflows.  There the reciprocal is infinite, the minimiser
                // infinite or not a number, the level clamped or the score not a number, which is never less than the best
                // so far -- such a coordinate is not chosen either way, and three instructions per coordinate are saved
                ci[v] = __builtin_amdgcn_rcpf(2.0f * a_c[c] * h[v]);
            } else {
                h[v] = hd[c * VEC + v];
                ci[v] = cinv[c * VEC + v];
            }
        }
    };

    int moves = 0, converged = 0, n_reduce = 0;
    uint32_t last_hi = kOrderedZero;

    // (ordered score, payload) of this lane's best candidate -> team-wide winner, uniform
    auto team_min = [&](float bs, float bu, int be, uint32_t flag) -> uint64_t {
        const int bi = (be / VEC) * STRIDE + tl * VEC + (be % VEC);
        const uint32_t payload = ((uint32_t)bi << 7) | ((uint32_t)((int)bu + 32) << 1) | flag;
        uint64_t key = wave_min_key(order_bits(bs), payload);
        if (W > 1) {
            const int p = n_reduce & 1;
            ++n_reduce;
            if (lane == 0) slots[p][wave] = key;
            __syncthreads();
#pragma unroll
            for (int w = 0; w < W; ++w) key = umin64(key, (uint64_t)slots[p][w]);
        }
        return key;
    };

    auto score_fast = [&]() -> uint64_t {
        float bs = 0.0f, bu = 0.0f, brf = 0.0f;
        int be = 0;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const float a = a_c[c];
            float hc[VEC], cc[VEC];
            diag_of(c, hc, cc);
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                const int e = c * VEC + v;
                const float qf = (float)((qpack[c] >> (8 * v)) & 0xffu);
                const float rf = fmaf(-g2[e], cc[v], qf);
                const float rn = __builtin_amdgcn_fmed3f(rintf(rf), 0.0f, top);
                const float u = rn - qf;
                const float d = a * u;
                const float s = d * fmaf(d, hc[v], g2[e]);
                if constexpr (LDSH && (E > 32 || E == 16)) {
                    // the compare and its four selects as one block: scheduled apart, the compiler keeps every coordinate's
                    // level change, minimiser and compare mask alive until the end of the chunk, and runs out of registers at 36
                    // per lane (30 spilled; none this way) and in the 64-register kernel for two columns per compute unit (19
                    // spilled, 9 this way; loop on 2048 x 16384 176 -> 167 ms).  The kernels in between fit as they are and lose 1 to
                    // 8 % to the wait state between the compare and the first select, so they keep the plain form.
                    asm volatile("v_cmp_nlt_f32 vcc, %4, %0\n\ts_nop 1\n\tv_cndmask_b32 %0, %4, %0, vcc\n\tv_cndmask_b32 %1, %5, %1, vcc\n\t"
                                 "v_cndmask_b32 %2, %6, %2, vcc\n\tv_cndmask_b32 %3, %7, %3, vcc"
                                 : "+v"(bs), "+v"(bu), "+v"(brf), "+v"(be) : "v"(s), "v"(u), "v"(rf), "n"(e) : "vcc");
                } else {
                    if (s < bs) { bs = s; bu = u; brf = rf; be = e; }
                }
            }
        }
        const float frac = brf - floorf(brf);
        const uint32_t flag = (fabsf(frac - 0.5f) < kHalfWindow) ? 1u : 0u;
        return team_min(bs, bu, be, flag);
    };

    auto score_exact = [&]() -> uint64_t {
        float bs = 0.0f, bu = 0.0f;
        int be = 0;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const float a = a_c[c];
            float hc[VEC], cc[VEC];
            diag_of(c, hc, cc);
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                const int e = c * VEC + v;
                const float qf = (float)((qpack[c] >> (8 * v)) & 0xffu);
                const float rf = __builtin_amdgcn_fmed3f(fmaf(-g2[e], cc[v], qf), 0.0f, top);
                const float r0 = floorf(rf), r1 = ceilf(rf);
                float u0 = r0 - qf;
                const float u1 = r1 - qf;
                const float d0 = a * u0, d1 = a * u1;
                float s0 = d0 * fmaf(d0, hc[v], g2[e]);
                const float s1 = d1 * fmaf(d1, hc[v], g2[e]);
                if constexpr (LDSH && (E > 32 || E == 16)) {
                    asm volatile("v_cmp_nlt_f32 vcc, %2, %0\n\ts_nop 1\n\tv_cndmask_b32 %0, %2, %0, vcc\n\tv_cndmask_b32 %1, %3, %1, vcc"
                                 : "+v"(s0), "+v"(u0) : "v"(s1), "v"(u1) : "vcc");      // equal scores keep the lower level
                    asm volatile("v_cmp_nlt_f32 vcc, %3, %0\n\ts_nop 1\n\tv_cndmask_b32 %0, %3, %0, vcc\n\tv_cndmask_b32 %1, %4, %1, vcc\n\t"
                                 "v_cndmask_b32 %2, %5, %2, vcc"
                                 : "+v"(bs), "+v"(bu), "+v"(be) : "v"(s0), "v"(u0), "n"(e) : "vcc");
                } else {
                    if (s1 < s0) { s0 = s1; u0 = u1; }      // equal scores keep the lower level
                    if (s0 < bs) { bs = s0; bu = u0; be = e; }
                }
            }
        }
        return team_min(bs, bu, be, 0u);
    };

    // A coordinate whose two neighbouring levels have the same loss to within the rounding of 2g can be moved up and down
    // for ever: both moves compute to a (tiny) negative score.  The paper's loop, and the oracle, go on to the end of the
    // budget.  So does this one, but not step by step: when a move undoes the previous one, 2g is written to the column's
    // row of the start gradient; if two moves later the codes are back (the two moves again undid each other) and 2g has
    // exactly the same bits, the state is that of two iterations ago, the loop is periodic from here on, and only the
    // parity of what is left of the budget matters.  Not done when the moves are traced.  Built into every kernel for 16-byte
    // chunks except the register kernels with 32 coordinates per lane (FF); the test reads the snapshot one chunk at a time, so
    // it costs no registers in the loop.
    auto team_all = [&](bool ok) -> bool {
        uint64_t v = (__ballot(ok) == ~0ull) ? 1u : 0u;
        if (W > 1) {
            const int p = n_reduce & 1;
            ++n_reduce;
            if (lane == 0) slots[p][wave] = v;
            __syncthreads();
#pragma unroll
            for (int w = 0; w < W; ++w) v = umin64(v, (uint64_t)slots[p][w]);
        }
        return v != 0;
    };
    uint32_t undo_move = 0xffffffffu;         // coordinate << 6 | (32 - level change) of the previous move: the move that would undo it
    int snap_t = -1;                          // iteration whose 2g the snapshot holds

    for (int t = 0; t < T; ++t) {
        if constexpr (LDSH) {
            tl = tid;
            asm volatile("" : "+v"(tl));
        }
        // ---- 1 + 2. score and arg-min
        uint64_t key = exact_only ? score_exact() : score_fast();
        uint32_t khi = __builtin_amdgcn_readfirstlane((uint32_t)(key >> 32));
        uint32_t klo = __builtin_amdgcn_readfirstlane((uint32_t)key);
        if (!exact_only && (khi >= kOrderedZero || (klo & 1u))) {
            key = score_exact();
            khi = __builtin_amdgcn_readfirstlane((uint32_t)(key >> 32));
            klo = __builtin_amdgcn_readfirstlane((uint32_t)key);
        }
        if (khi >= kOrderedZero) { converged = 1; break; }     // no move lowers the loss
        const int istar = (int)(klo >> 7);
        const int ustar = (int)((klo >> 1) & 63u) - 32;
        // ---- 3. commit: code, then gradient
        const int gstar = (n_grp == 1) ? 0 : (group_shift >= 0 ? (istar >> group_shift) : (istar / group));
        const float delta2 = 2.0f * (scale_j[gstar] * (float)ustar);
        const float4* hrow4 = reinterpret_cast<const float4*>(H + (int64_t)istar * d_in);
        const float* hrow = H + (int64_t)istar * d_in;

        const int cstar = istar / STRIDE;
        const int within = istar - cstar * STRIDE;
        const uint32_t inc = (within / VEC == tl) ? ((uint32_t)ustar << (8 * (within % VEC))) : 0u;
#pragma unroll
        for (int c = 0; c < NCH; ++c) qpack[c] += (c == cstar) ? inc : 0u;

        // all loads of the row first (lanes past the end read the row's start and add nothing), so that the
        // chunks' memory latencies overlap instead of following one another
        if constexpr (VEC == 4) {
            constexpr int BATCH = NCH;        // chunks whose loads are in flight together: all of them
#pragma unroll
            for (int c0 = 0; c0 < NCH; c0 += BATCH) {
                float4 hv[BATCH];
#pragma unroll
                for (int cb = 0; cb < BATCH; ++cb) {
                    const int c = c0 + cb;
                    if (c < NCH) {
                        const int base = c * STRIDE + tl * VEC;
                        hv[cb] = hrow4[(base < d_in ? base : 0) >> 2];
                    }
                }
#pragma unroll
                for (int cb = 0; cb < BATCH; ++cb) {
                    const int c = c0 + cb;
                    if (c < NCH) {
                        const float m = (c * STRIDE + tl * VEC < d_in) ? delta2 : 0.0f;
                        g2[c * 4 + 0] = fmaf(m, hv[cb].x, g2[c * 4 + 0]);
                        g2[c * 4 + 1] = fmaf(m, hv[cb].y, g2[c * 4 + 1]);
                        g2[c * 4 + 2] = fmaf(m, hv[cb].z, g2[c * 4 + 2]);
                        g2[c * 4 + 3] = fmaf(m, hv[cb].w, g2[c * 4 + 3]);
                    }
                }
            }
        } else {
            float hv[NCH];
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const int base = c * STRIDE + tid;
                hv[c] = hrow[base < d_in ? base : 0];
            }
#pragma unroll
            for (int c = 0; c < NCH; ++c) g2[c] = fmaf((c * STRIDE + tid < d_in) ? delta2 : 0.0f, hv[c], g2[c]);
        }
        if (trace != nullptr && tid == 0 && moves < trace_cap) trace[j * trace_cap + moves] = (int32_t)(klo >> 1);
        last_hi = khi;
        ++moves;
        // ---- the same coordinate moved back: snapshot, or compare with the snapshot of two iterations ago (uniform branches).
        // Two moves that undo each other restore the codes whatever came before, so the comparison of 2g is the whole test.
        const uint32_t this_move = FF ? (klo >> 1) : 0u;
        if (FF && __builtin_expect(this_move == undo_move, 0) && trace == nullptr) {      // rare: kept out of the straight path
            float* snap = G0 + j * (int64_t)d_in;                        // the start gradient is not needed any more
            bool take = !(snap_t >= 0 && t == snap_t + 1);               // keep the snapshot for the comparison one move on
            if (snap_t >= 0 && t == snap_t + 2) {
                bool same = true;
#pragma unroll
                for (int c = 0; c < NCH; ++c) {
                    const int base = c * STRIDE + tl * VEC;
                    if (base < d_in) {
#pragma unroll
                        for (int v = 0; v < VEC; ++v) same &= __float_as_uint(snap[base + v]) == __float_as_uint(g2[c * VEC + v]);
                    }
                    __builtin_amdgcn_sched_barrier(0);       // one chunk of the snapshot in registers at a time: this path is rare
                }
                if (team_all(same)) {                                    // periodic from here: only the parity of the rest matters
                    const int left = T - (t + 1);
                    moves += left & ~1;
                    T = t + 1 + (left & 1);
                    take = false;
                }
            }
            if (take) {
#pragma unroll
                for (int c = 0; c < NCH; ++c) {
                    const int base = c * STRIDE + tl * VEC;
                    if (base < d_in) {
#pragma unroll
                        for (int v = 0; v < VEC; ++v) snap[base + v] = g2[c * VEC + v];
                    }
                }
                snap_t = t;
            }
        }
        if (FF) undo_move = (this_move & ~63u) | (64u - (this_move & 63u));
    }

    // ---- write back
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int base = c * STRIDE + tid * VEC;
        if (base < d_in) {
            if (VEC == 4) *reinterpret_cast<uint32_t*>(Qj + base) = qpack[c];
            else Qj[base] = (uint8_t)qpack[c];
            if (G_out != nullptr) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) G_out[j * (int64_t)d_in + base + v] = 0.5f * g2[c * VEC + v];
            }
        }
    }
    if (stats != nullptr && tid == 0) {
        cdq_col_stats s;
        s.moves = moves;
        s.iters = moves + converged;
        s.converged = converged;
        s.last_score = moves ? unorder_bits(last_hi) : 0.0f;
        stats[j] = s;
    }
}

template <int W, int E, int VEC, bool LDSH, bool FF>
__global__ __launch_bounds__(64 * W) void cd_fused_kernel(
    const float* __restrict__ H, const float* __restrict__ hdiag, float* G0,
    const float* __restrict__ scale, uint8_t* __restrict__ Q, int d_in, int bits, int group, int group_shift,
    int n_grp, int T, int exact_only, cdq_col_stats* __restrict__ stats, int32_t* __restrict__ trace,
    int64_t trace_cap, float* __restrict__ G_out) {
    cd_fused_body<W, E, VEC, LDSH, FF>(H, hdiag, G0, scale, Q, d_in, bits, group, group_shift, n_grp, T, exact_only, stats, trace,
                                       trace_cap, G_out);
}

// Two columns per CU for d_in up to 16384: the diagonal in LDS (64 KiB per column) and the kernel held to 64 registers, so
// that two teams of 16 wavefronts are resident and one column's scoring runs while the other waits for its row of H.
template <int E, bool FF>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(8, 8))) void cd_fused_pair_kernel(
    const float* __restrict__ H, const float* __restrict__ hdiag, float* G0,
    const float* __restrict__ scale, uint8_t* __restrict__ Q, int d_in, int bits, int group, int group_shift,
    int n_grp, int T, int exact_only, cdq_col_stats* __restrict__ stats, int32_t* __restrict__ trace,
    int64_t trace_cap, float* __restrict__ G_out) {
    cd_fused_body<16, E, 4, true, FF>(H, hdiag, G0, scale, Q, d_in, bits, group, group_shift, n_grp, T, exact_only, stats, trace,
                                      trace_cap, G_out);
}

__global__ __launch_bounds__(256) void extract_diag_kernel(const float* __restrict__ H, int64_t d_in, float* __restrict__ hdiag) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < d_in) hdiag[i] = H[i * d_in + i];
}

template <int W, int E, int VEC, bool LDSH = false>
int launch_one(const float* H, const float* hdiag, float* G0, const float* scale, uint8_t* Q, int64_t d_out,
               int d_in, int bits, int group, int group_shift, int n_grp, int T, int exact_only, cdq_col_stats* stats,
               int32_t* trace, int64_t trace_cap, float* G_out, hipStream_t st) {
    constexpr bool FF = (VEC == 4 && (E <= 24 || LDSH));
    const size_t lds = LDSH ? sizeof(float) * 64 * W * E : 0;
    if (LDSH) {
        static const hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void*>(cd_fused_kernel<W, E, VEC, LDSH, FF>),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (rc != hipSuccess) return CDQ_EHIP;
    }
    hipLaunchKernelGGL((cd_fused_kernel<W, E, VEC, LDSH, FF>), dim3((unsigned)d_out), dim3(64 * W), lds, st, H, hdiag, G0, scale, Q, d_in,
                       bits, group, group_shift, n_grp, T, exact_only, stats, trace, trace_cap, G_out);
    CDQ_LAUNCH_CHECK();
    return CDQ_OK;
}

}  // namespace

int extract_diag_launch(const float* H, int64_t d_in, float* hdiag, hipStream_t st) {
    hipLaunchKernelGGL(extract_diag_kernel, dim3((unsigned)((d_in + 255) / 256)), dim3(256), 0, st, H, d_in, hdiag);
    CDQ_LAUNCH_CHECK();
    return CDQ_OK;
}

// Launch shape: a team of `waves` wavefronts per column, `elems` coordinates per lane.
// Measured on MI355X: 16 coordinates per lane is the best trade between the serial scoring chain
// of a lane, registers (occupancy) and the cost of the cross-wavefront step, for every d_in from
// 2048 to 16384; beyond that 24, 32 or 36 per lane on 16 wavefronts with the Hessian diagonal in LDS.  With few columns the chain is split
// over more wavefronts so the 256 CUs x 4 SIMDs still have work in flight.
// `aligned16`: rows of H start on 16-byte and rows of Q on 4-byte boundaries, so 16-byte chunks can be used.
int cd_choose_shape(int64_t d_out, int64_t d_in, int64_t group, bool aligned16, int* waves, int* elems, int* vec) {
    const int v = (aligned16 && d_in % 4 == 0 && group % 4 == 0) ? 4 : 1;
    auto team = [&](int e) {
        const int64_t need = (d_in + 64 * (int64_t)e - 1) / (64 * (int64_t)e);
        int w = 1;
        while (w < need) w <<= 1;
        return w;
    };
    int e = (d_in <= 1024) ? 8 : 16;
    int w = team(e);
    if (w > 16) {
        e = (v == 4 && d_in <= 64 * 16 * 24) ? 24 : 32;
        w = team(e);
        if (w > 16) {                          // beyond 32768: 36 per lane with the Hessian diagonal in LDS (16-byte chunks only)
            e = 36;
            w = 16;
            if (v != 4 || d_in > (int64_t)64 * w * e) return CDQ_EUNSUPPORTED;
        }
    }
    while (e > 4 && e <= 32 && e != 24 && d_out * w < 2048 && team(e / 2) <= 8) {
        e /= 2;
        w = team(e);
    }
    *waves = w;
    *elems = e;
    *vec = v;
    return CDQ_OK;
}

// Columns resident per compute unit: two for the 16 x 16 shape once the layer has more columns than the chip has compute
// units (measured on 2048 x 16384: loop 184 -> 165 ms), one otherwise.
int cd_choose_teams(int64_t d_out, int waves, int elems, int vec) {
    return (waves == 16 && elems == 16 && vec == 4 && d_out > 256) ? 2 : 1;
}

#define CDQ_CD_CASE(Wv, Ev)                                                                                        \
    if (waves == Wv && elems == Ev) {                                                                              \
        return vec == 4 ? launch_one<Wv, Ev, 4>(H, hdiag, G0, scale, Q, d_out, di, bits, gr, gshift, ng, Ti, exact_only, \
                                                stats, trace, trace_cap, G_out, st)                                \
                        : launch_one<Wv, Ev, 1>(H, hdiag, G0, scale, Q, d_out, di, bits, gr, gshift, ng, Ti, exact_only, \
                                                stats, trace, trace_cap, G_out, st);                               \
    }

int cd_launch(const float* H, const float* hdiag, float* G0, const float* scale, uint8_t* Q, int64_t d_out,
              int64_t d_in, int bits, int64_t group, int64_t T, cdq_col_stats* stats, int waves, int elems, int vec,
              int exact_only, int32_t* trace, int64_t trace_cap, float* G_out, hipStream_t st, int teams_per_cu) {
    if (d_out == 0) return CDQ_OK;
    const bool pair_shape = waves == 16 && elems == 16 && vec == 4;
    if (teams_per_cu < 0 || teams_per_cu > 2 || (teams_per_cu == 2 && !pair_shape)) return CDQ_EINVAL;
    if (teams_per_cu == 0) teams_per_cu = cd_choose_teams(d_out, waves, elems, vec);
    if ((int64_t)64 * waves * elems < d_in) return CDQ_EINVAL;
    if (d_out > 0x7fffffffLL || d_in > CDQ_MAX_D_IN) return CDQ_EUNSUPPORTED;
    const int di = (int)d_in, gr = (int)group, ng = (int)(d_in / group);
    const int Ti = (int)(T > 0x7fffffffLL ? 0x7fffffffLL : T);
    int gshift = -1;
    if ((group & (group - 1)) == 0) {
        gshift = 0;
        while (((int64_t)1 << gshift) < group) ++gshift;
    }
    // 16 wavefronts with more than 16 coordinates per lane do not fit the 128 registers a lane has there without spilling
    // in the loop (measured at d_in = 24576: 19 us per update); the variant with the Hessian diagonal in LDS does, or nearly
    if (pair_shape && teams_per_cu == 2) {
        const size_t lds = sizeof(float) * 64 * 16 * 16;
        static const hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void*>(cd_fused_pair_kernel<16, true>),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (rc != hipSuccess) return CDQ_EHIP;
        hipLaunchKernelGGL((cd_fused_pair_kernel<16, true>), dim3((unsigned)d_out), dim3(1024), lds, st, H, hdiag, G0, scale, Q, di, bits, gr,
                           gshift, ng, Ti, exact_only, stats, trace, trace_cap, G_out);
        CDQ_LAUNCH_CHECK();
        return CDQ_OK;
    }
    if (waves == 16 && elems == 24 && vec == 4)
        return launch_one<16, 24, 4, true>(H, hdiag, G0, scale, Q, d_out, di, bits, gr, gshift, ng, Ti, exact_only, stats, trace,
                                           trace_cap, G_out, st);
    if (waves == 16 && elems == 32 && vec == 4)
        return launch_one<16, 32, 4, true>(H, hdiag, G0, scale, Q, d_out, di, bits, gr, gshift, ng, Ti, exact_only, stats, trace,
                                           trace_cap, G_out, st);
    CDQ_CD_CASE(1, 4) CDQ_CD_CASE(1, 8) CDQ_CD_CASE(1, 16) CDQ_CD_CASE(1, 32)
    CDQ_CD_CASE(2, 4) CDQ_CD_CASE(2, 8) CDQ_CD_CASE(2, 16) CDQ_CD_CASE(2, 32)
    CDQ_CD_CASE(4, 4) CDQ_CD_CASE(4, 8) CDQ_CD_CASE(4, 16) CDQ_CD_CASE(4, 32)
    CDQ_CD_CASE(8, 4) CDQ_CD_CASE(8, 8) CDQ_CD_CASE(8, 16) CDQ_CD_CASE(8, 32)
    CDQ_CD_CASE(16, 4) CDQ_CD_CASE(16, 8) CDQ_CD_CASE(16, 16) CDQ_CD_CASE(16, 32)
    if (waves == 16 && elems == 36 && vec == 4)
        return launch_one<16, 36, 4, true>(H, hdiag, G0, scale, Q, d_out, di, bits, gr, gshift, ng, Ti, exact_only, stats, trace,
                                           trace_cap, G_out, st);
    return CDQ_EINVAL;
}

}  // namespace cdq
