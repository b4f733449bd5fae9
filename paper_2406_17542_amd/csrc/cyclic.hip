// Cyclic (fixed-order) coordinate descent: the variant without the arg-min over coordinates that the
// paper contrasts greedy CD with (Section 1; appendix comparison with QuantEase).  Visit t handles
// coordinate t mod d_in: every level r is scored, delta = a (r - q_i), s = delta * fma(delta, H_ii, 2 g_i),
// and the first strict minimum is committed if negative: 2g <- fma(2 delta, H[i,:], 2g).
// One workgroup owns a column; 2g, H_ii and the codes sit in LDS.  Between two moves the gradient does
// not change, so the next `blockDim` visits are scored at once, one per thread, and the first of them
// that moves is the one the sequential order would take; everything after it is rescored.  A column
// stops once d_in consecutive visits made no move.
#include "cdq_internal.h"

namespace cdq {
namespace {

template <int BITS>
__global__ __launch_bounds__(256) void cyclic_cd_kernel(const float* __restrict__ H, const float* __restrict__ hdiag,
                                                        const float* __restrict__ G0, const float* __restrict__ scale,
                                                        uint8_t* __restrict__ Q, int d_in, int group, int64_t T,
                                                        cdq_col_stats* __restrict__ stats, float* __restrict__ G_out,
                                                        int32_t* __restrict__ trace, int trace_cap) {
    constexpr int L = 1 << BITS;
    constexpr int NT = 256;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_grp = d_in / group;
    const int64_t j = blockIdx.x;
    float* g2 = reinterpret_cast<float*>(smem);          // [d_in]
    float* hd = g2 + d_in;                               // [d_in]
    float* a = hd + d_in;                                // [n_grp]
    int* first = reinterpret_cast<int*>(a + n_grp);      // [2][4] first mover of each wavefront, double-buffered
    float* commit = reinterpret_cast<float*>(first + 8); // [2][2] 2 delta, score
    int* commit_r = reinterpret_cast<int*>(commit + 4);  // [2]
    uint8_t* q = reinterpret_cast<uint8_t*>(commit_r + 2);   // [d_in]

    for (int c = tid; c < d_in; c += NT) {
        g2[c] = 2.0f * G0[j * (int64_t)d_in + c];
        hd[c] = hdiag[c];
        q[c] = Q[j * (int64_t)d_in + c];
    }
    for (int i = tid; i < n_grp; i += NT) a[i] = scale[j * n_grp + i];
    __syncthreads();

    int64_t t = 0;
    int idle = 0, moves = 0, converged = 0, round = 0;
    float last_s = 0.0f;
    while (t < T) {
        if (idle >= d_in) { converged = 1; break; }
        // visits t .. t+window-1, never the same coordinate twice, never past T or past the idle limit
        int64_t window = NT;
        if (window > T - t) window = T - t;
        if (window > d_in - idle) window = d_in - idle;
        float best_s = 0.0f, best_d = 0.0f;
        int best_r = -1;
        const int i = (int)((t + tid) % d_in);
        if (tid < window) {
            const float ai = a[i / group], hii = hd[i], gi = g2[i];
            const int qi = q[i];
#pragma unroll
            for (int r = 0; r < L; ++r) {
                const float d = ai * (float)(r - qi);
                const float s = d * fmaf(d, hii, gi);
                if (s < best_s) { best_s = s; best_r = r; best_d = d; }
            }
        }
        const unsigned long long m = __ballot(best_r >= 0);
        int* slot = first + (round & 1) * 4;
        if (lane == 0) slot[wave] = m ? wave * 64 + __builtin_ctzll(m) : 0x7fffffff;
        __syncthreads();
        const int mover = min(min(slot[0], slot[1]), min(slot[2], slot[3]));
        if (mover == 0x7fffffff) {                       // nobody in the window moves
            t += window;
            idle += (int)window;
            ++round;
            continue;
        }
        float* cm = commit + (round & 1) * 2;
        if (tid == mover) {
            cm[0] = 2.0f * best_d;
            cm[1] = best_s;
            commit_r[round & 1] = best_r;
            q[i] = (uint8_t)best_r;
            if (trace != nullptr && moves < trace_cap) trace[j * trace_cap + moves] = (i << 7) | best_r;
        }
        __syncthreads();
        const int istar = (int)((t + mover) % d_in);
        const float d2 = cm[0];
        last_s = cm[1];
        const float* hrow = H + (int64_t)istar * d_in;
        for (int c = 4 * tid; c < d_in; c += 4 * NT) {
            const float4 h = *reinterpret_cast<const float4*>(hrow + c);
            float4 g = *reinterpret_cast<float4*>(g2 + c);
            g.x = fmaf(d2, h.x, g.x); g.y = fmaf(d2, h.y, g.y); g.z = fmaf(d2, h.z, g.z); g.w = fmaf(d2, h.w, g.w);
            *reinterpret_cast<float4*>(g2 + c) = g;
        }
        __syncthreads();
        t += mover + 1;
        idle = 0;
        ++moves;
        ++round;
    }
    if (!converged && idle >= d_in) converged = 1;
    __syncthreads();
    for (int c = tid; c < d_in; c += NT) {
        Q[j * (int64_t)d_in + c] = q[c];
        if (G_out != nullptr) G_out[j * (int64_t)d_in + c] = 0.5f * g2[c];
    }
    if (tid == 0 && stats != nullptr) {
        cdq_col_stats s;
        s.moves = moves;
        s.iters = (int32_t)(t > 0x7fffffffLL ? 0x7fffffffLL : t);
        s.converged = converged;
        s.last_score = last_s;
        stats[j] = s;
    }
}

size_t cyclic_lds_bytes(int64_t d_in, int64_t group) {
    return cdq_align_up(sizeof(float) * (2 * d_in + d_in / group) + sizeof(int) * 8 + sizeof(float) * 4 + sizeof(int) * 2 + (size_t)d_in, 16);
}

}  // namespace

// workspace: G0 [d_out][d_in] fp32 | hdiag [d_in]
size_t cyclic_workspace_bytes(int64_t d_out, int64_t d_in) {
    return cdq_align_up((size_t)d_out * d_in * sizeof(float), 256) + cdq_align_up((size_t)d_in * sizeof(float), 256);
}

int cyclic_launch(const float* H, const float* Wt, const float* scale, const float* zero, uint8_t* Q, int64_t d_out, int64_t d_in,
                  int bits, int64_t group, int64_t T, cdq_col_stats* stats, float* G_out, int32_t* trace, int64_t trace_cap,
                  void* ws, size_t ws_bytes, hipStream_t st) {
    if (d_out == 0) return CDQ_OK;
    const size_t lds = cyclic_lds_bytes(d_in, group);
    if (lds > 160 * 1024 || d_in % 4 != 0 || ((uintptr_t)H & 15) || d_in >= (1 << 24) || d_out > 0x7fffffffLL) return CDQ_EUNSUPPORTED;
    if (ws == nullptr || ((uintptr_t)ws & 255) || ws_bytes < cyclic_workspace_bytes(d_out, d_in)) return CDQ_EWORKSPACE;
    float* G0 = (float*)ws;
    float* hdiag = (float*)((char*)ws + cdq_align_up((size_t)d_out * d_in * sizeof(float), 256));
    int rc = gradient_launch(H, Wt, scale, zero, Q, d_out, d_in, group, G0, st);
    if (rc != CDQ_OK) return rc;
    rc = extract_diag_launch(H, d_in, hdiag, st);
    if (rc != CDQ_OK) return rc;
    const int cap = (int)(trace_cap > 0x7fffffffLL ? 0x7fffffffLL : trace_cap);
#define CYC_CASE(B)                                                                                                               \
    case B:                                                                                                                       \
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(cyclic_cd_kernel<B>), hipFuncAttributeMaxDynamicSharedMemorySize,   \
                                (int)lds) != hipSuccess)                                                                          \
            return CDQ_EHIP;                                                                                                      \
        hipLaunchKernelGGL((cyclic_cd_kernel<B>), dim3((unsigned)d_out), dim3(256), lds, st, H, (const float*)hdiag,              \
                           (const float*)G0, scale, Q, (int)d_in, (int)group, T, stats, G_out, trace, cap);                       \
        break;
    switch (bits) {
        CYC_CASE(2) CYC_CASE(3) CYC_CASE(4)
        default: return CDQ_EINVAL;
    }
#undef CYC_CASE
    CDQ_LAUNCH_CHECK();
    return CDQ_OK;
}

}  // namespace cdq
