// One iteration of Algorithm 1 as two separate kernels over gradients kept in global memory:
//   score_argmin : the arg-min step  (per column: best coordinate, level and score)
//   gather_update: the code-update and gradient-update steps for the selected coordinates
// They are the general form of the loop -- any d_in, one launch pair per iteration -- and make
// each step checkable on its own.  The fused kernel (cd_fused.hip) is the fast path; it keeps
// the same state in registers and never writes the gradient back.
#include "cdq_internal.h"
#include "wave_min.h"

namespace cdq {
namespace {

constexpr uint32_t kNoMove = kOrderedZero;

// one workgroup per column; key = (ordered score, coordinate, level)
__global__ __launch_bounds__(256) void score_argmin_kernel(const float* __restrict__ hdiag, const float* __restrict__ scale,
                                                           const uint8_t* __restrict__ Q, const float* __restrict__ G,
                                                           int64_t d_in, int bits, int64_t group, int64_t n_grp,
                                                           int32_t* __restrict__ out_i, int32_t* __restrict__ out_r,
                                                           float* __restrict__ out_s) {
    __shared__ unsigned long long red[4];
    const int64_t j = blockIdx.x;
    const float top = (float)((1 << bits) - 1);
    const uint8_t* q = Q + j * d_in;
    const float* g = G + j * d_in;
    const float* a_j = scale + j * n_grp;
    uint64_t key = ((uint64_t)kNoMove << 32) | 0xffffffffu;
    for (int64_t i = threadIdx.x; i < d_in; i += 256) {
        const float a = a_j[i / group], h = hdiag[i], g2 = 2.0f * g[i], qf = (float)q[i];
        // the score is a convex parabola in the level: its integer minimum is floor or ceil of the
        // clamped continuous minimiser; both are scored with the canonical formula
        float rf = qf;
        if (h > 0.0f) rf = fmaf(-g2, fminf(__frcp_rn(2.0f * a * h), 3.0e38f), qf);
        rf = __builtin_amdgcn_fmed3f(rf, 0.0f, top);
        const float r0 = floorf(rf), r1 = ceilf(rf);
        const float d0 = a * (r0 - qf), d1 = a * (r1 - qf);
        const float s0 = d0 * fmaf(d0, h, g2), s1 = d1 * fmaf(d1, h, g2);
        const bool take1 = s1 < s0;                       // equal scores keep the lower level
        const float s = take1 ? s1 : s0;
        const uint32_t r = (uint32_t)(take1 ? r1 : r0);
        key = umin64(key, ((uint64_t)order_bits(s) << 32) | ((uint32_t)i << 4) | r);
    }
    for (int o = 32; o; o >>= 1) key = umin64(key, (uint64_t)__shfl_xor((unsigned long long)key, o));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = key;
    __syncthreads();
    if (threadIdx.x == 0) {
        key = umin64(umin64(red[0], red[1]), umin64(red[2], red[3]));
        const uint32_t hi = (uint32_t)(key >> 32), lo = (uint32_t)key;
        if (hi >= kNoMove) {
            out_i[j] = -1; out_r[j] = -1; out_s[j] = 0.0f;
        } else {
            out_i[j] = (int32_t)(lo >> 4); out_r[j] = (int32_t)(lo & 15u); out_s[j] = __uint_as_float(~hi);
        }
    }
}

// one workgroup per column: commit the selected move, if any
__global__ __launch_bounds__(256) void gather_update_kernel(const float* __restrict__ H, const float* __restrict__ scale,
                                                            uint8_t* __restrict__ Q, float* __restrict__ G, int64_t d_in,
                                                            int64_t group, int64_t n_grp, const int32_t* __restrict__ sel_i,
                                                            const int32_t* __restrict__ sel_r, int32_t* __restrict__ moves) {
    const int64_t j = blockIdx.x;
    const int32_t i = sel_i[j];
    if (i < 0) return;                                     // converged column: nothing to do
    const int32_t r = sel_r[j];
    const int q_old = Q[j * d_in + i];
    const float delta = scale[j * n_grp + i / group] * (float)(r - q_old);
    const float* hrow = H + (int64_t)i * d_in;             // H symmetric: row i is column i
    float* g = G + j * d_in;
    for (int64_t k = threadIdx.x; k < d_in; k += 256) g[k] = fmaf(delta, hrow[k], g[k]);
    __syncthreads();                                       // every lane has read the old code
    if (threadIdx.x == 0) {
        Q[j * d_in + i] = (uint8_t)r;
        if (moves != nullptr) moves[j] += 1;
    }
}

}  // namespace

int score_argmin_launch(const float* hdiag, const float* scale, const uint8_t* Q, const float* G, int64_t d_out, int64_t d_in,
                        int bits, int64_t group, int32_t* out_i, int32_t* out_r, float* out_s, hipStream_t st) {
    if (d_out == 0) return CDQ_OK;
    if (d_out > 0x7fffffffLL || d_in >= (1LL << 28)) return CDQ_EUNSUPPORTED;
    hipLaunchKernelGGL(score_argmin_kernel, dim3((unsigned)d_out), dim3(256), 0, st, hdiag, scale, Q, G, d_in, bits, group,
                       d_in / group, out_i, out_r, out_s);
    CDQ_LAUNCH_CHECK();
    return CDQ_OK;
}

int gather_update_launch(const float* H, const float* scale, uint8_t* Q, float* G, int64_t d_out, int64_t d_in, int64_t group,
                         const int32_t* sel_i, const int32_t* sel_r, int32_t* moves, hipStream_t st) {
    if (d_out == 0) return CDQ_OK;
    if (d_out > 0x7fffffffLL) return CDQ_EUNSUPPORTED;
    hipLaunchKernelGGL(gather_update_kernel, dim3((unsigned)d_out), dim3(256), 0, st, H, scale, Q, G, d_in, group, d_in / group,
                       sel_i, sel_r, moves);
    CDQ_LAUNCH_CHECK();
    return CDQ_OK;
}

}  // namespace cdq
