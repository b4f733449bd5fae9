// Order-preserving keys for candidate scores and a wavefront-wide lexicographic minimum.
// Shared by the kernels that pick the move with the smallest score (greedy CD, block CD).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cdq {
namespace {

constexpr uint32_t kOrderedZero = 0x80000000u;   // image of "no improving move"
// Order-preserving image of a candidate score.  Only strictly negative scores are moves; a zero
// of either sign (0 * g has the sign of g) and anything positive mean "no move".
__device__ __forceinline__ uint32_t order_bits(float s) {
    return (s < 0.0f) ? ~__float_as_uint(s) : kOrderedZero;
}
__device__ __forceinline__ float unorder_bits(uint32_t o) {
    return __uint_as_float((o & 0x80000000u) ? (o & 0x7fffffffu) : ~o);
}
__device__ __forceinline__ uint32_t umin32(uint32_t a, uint32_t b) { return a < b ? a : b; }
__device__ __forceinline__ uint64_t umin64(uint64_t a, uint64_t b) { return a < b ? a : b; }

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_min(uint32_t v) {
    const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xF, 0xF, false);
    return umin32(v, o);
}

// Minimum of (k32, payload) in lexicographic order over one wavefront; the result is uniform.
__device__ __forceinline__ uint64_t wave_min_key(uint32_t k32, uint32_t payload) {
    uint32_t m = k32;
    m = dpp_min<0xB1>(m);     // quad_perm [1,0,3,2]
    m = dpp_min<0x4E>(m);     // quad_perm [2,3,0,1]
    m = dpp_min<0x141>(m);    // row_half_mirror
    m = dpp_min<0x140>(m);    // row_mirror: every lane of a 16-lane row now holds the row minimum
    const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)m, 0), r1 = (uint32_t)__builtin_amdgcn_readlane((int)m, 16);
    const uint32_t r2 = (uint32_t)__builtin_amdgcn_readlane((int)m, 32), r3 = (uint32_t)__builtin_amdgcn_readlane((int)m, 48);
    const uint32_t best = umin32(umin32(r0, r1), umin32(r2, r3));
    uint32_t pay = 0xffffffffu;
    if (best < kOrderedZero) {
        unsigned long long tied = __ballot(k32 == best);
        do {                                  // almost always a single lane
            const int l = __builtin_ctzll(tied);
            pay = umin32(pay, (uint32_t)__builtin_amdgcn_readlane((int)payload, l));
            tied &= tied - 1;
        } while (tied);
    }
    return ((uint64_t)best << 32) | pay;
}

}  // namespace
}  // namespace cdq
