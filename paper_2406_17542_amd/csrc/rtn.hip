// MinMax grid + round-to-nearest codes: Eq. (2) of the paper with clipping strength 1,
// per (output column, group).  One wavefront owns one (column, group) pair.
#include "cdq_internal.h"

namespace cdq {

namespace {

__device__ __forceinline__ float wave_min(float v) {
    for (int o = 32; o; o >>= 1) v = fminf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
    for (int o = 32; o; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}

__global__ __launch_bounds__(256) void rtn_kernel(const float* __restrict__ Wt, int64_t d_out, int64_t d_in,
                                                  int bits, int64_t group, int64_t n_grp,
                                                  float* __restrict__ scale, float* __restrict__ zero,
                                                  uint8_t* __restrict__ Q) {
    const int lane = threadIdx.x & 63;
    const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (item >= d_out * n_grp) return;
    const int64_t j = item / n_grp, gi = item % n_grp;
    const float* w = Wt + j * d_in + gi * group;
    uint8_t* q = Q + j * d_in + gi * group;

    // 16-byte loads and 4-byte code stores where the group allows it (same arithmetic per element either way)
    const bool vec4 = group % 4 == 0 && ((uintptr_t)w & 15) == 0 && ((uintptr_t)q & 3) == 0;
    const int n4 = (int)(group / 4);
    float lo = INFINITY, hi = -INFINITY;
    if (vec4) {
        for (int k = lane; k < n4; k += 64) {
            const float4 v = reinterpret_cast<const float4*>(w)[k];
            lo = fminf(fminf(lo, v.x), fminf(v.y, fminf(v.z, v.w)));
            hi = fmaxf(fmaxf(hi, v.x), fmaxf(v.y, fmaxf(v.z, v.w)));
        }
    } else {
        for (int64_t k = lane; k < group; k += 64) {
            const float v = w[k];
            lo = fminf(lo, v);
            hi = fmaxf(hi, v);
        }
    }
    lo = wave_min(lo);
    hi = wave_max(hi);

    const float top = (float)((1 << bits) - 1);
    float a = __fdiv_rn(hi - lo, top);
    if (!(a > 0.0f) || isinf(a)) a = 1.0f;      // constant group: any scale reproduces w with code 0
    if (lane == 0) {
        scale[item] = a;
        zero[item] = lo;
    }
    auto code = [&](float x) -> uint32_t {
        const float t = __fdiv_rn(x - lo, a);
        return (uint32_t)fminf(fmaxf(rintf(t), 0.0f), top);      // rintf: round half to even
    };
    if (vec4) {
        for (int k = lane; k < n4; k += 64) {
            const float4 v = reinterpret_cast<const float4*>(w)[k];
            reinterpret_cast<uint32_t*>(q)[k] = code(v.x) | (code(v.y) << 8) | (code(v.z) << 16) | (code(v.w) << 24);
        }
    } else {
        for (int64_t k = lane; k < group; k += 64) q[k] = (uint8_t)code(w[k]);
    }
}

}  // namespace

int rtn_launch(const float* Wt, int64_t d_out, int64_t d_in, int bits, int64_t group,
               float* scale, float* zero, uint8_t* Q, hipStream_t st) {
    const int64_t n_grp = d_in / group;
    const int64_t items = d_out * n_grp;
    if (items == 0) return CDQ_OK;
    const int64_t blocks = (items + 3) / 4;
    if (blocks > 0x7fffffffLL) return CDQ_EUNSUPPORTED;
    hipLaunchKernelGGL(rtn_kernel, dim3((unsigned)blocks), dim3(256), 0, st, Wt, d_out, d_in, bits, group, n_grp,
                       scale, zero, Q);
    CDQ_LAUNCH_CHECK();
    return CDQ_OK;
}

}  // namespace cdq
