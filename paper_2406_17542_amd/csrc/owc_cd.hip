// OWC-CD (paper Algorithm 3): greedy coordinate descent over the clipping strengths of the groups
// of a sub-channel grid (Section 3.2, "Initialization").  One workgroup owns one output column for
// all T iterations; its state lives in LDS:
//   w, e (current residual a q + b - w, fp32), v = 2 H e (fp64), the grid's scales a(i,k),
//   quad(i,k) = d^T H_ii d for d = e(i,k) - e_cur(i)   (fp64, cached: it only changes for the
//   group whose clipping strength moved), and the residuals e(i*,k) of one group at a time.
// Per iteration: score(i,k) = quad(i,k) + v_i^T d(i,k) for all groups i and grid points k,
// arg-min (ties: group, then grid index), and if negative: v += 2 H[:, group i*] d*, e <- e(i*,k*),
// quad(i*, .) recomputed.  Every sum is fp64 so that it agrees with any other summation order to
// ~1e-16; Eq. (2) and the residual are the same fp32 operations as in the round-to-nearest kernel.
// The algorithm box of the paper initialises v with a minus sign that contradicts its own update
// line; v = +2He makes the score the exact loss change and is what is used.
#include "cdq_internal.h"

namespace cdq {
namespace {

__device__ __forceinline__ float owc_scale(float lo, float hi, int k, int n_gamma, float top) {
    const float gamma = __fdiv_rn((float)k, (float)n_gamma);
    float a = __fdiv_rn(gamma * (hi - lo), top);
    if (!(a > 0.0f) || isinf(a)) a = 1.0f;
    return a;
}
__device__ __forceinline__ float owc_code(float w, float lo, float a, float top) {
    return fminf(fmaxf(rintf(__fdiv_rn(w - lo, a)), 0.0f), top);
}
__device__ __forceinline__ float owc_resid(float w, float lo, float a, float top) {
    return fmaf(a, owc_code(w, lo, a, top), lo) - w;
}

struct OwcBest { double s; int p; };
__device__ __forceinline__ OwcBest owc_min(OwcBest x, OwcBest y) {
    return (y.s < x.s || (y.s == x.s && y.p < x.p)) ? y : x;
}

__global__ __launch_bounds__(256) void owc_cd_kernel(const float* __restrict__ H, const float* __restrict__ Wt, int d_in,
                                                     int bits, int group, int n_gamma, int T, float* __restrict__ scale,
                                                     float* __restrict__ zero, uint8_t* __restrict__ Q,
                                                     int32_t* __restrict__ gamma_idx, int32_t* __restrict__ moves_out,
                                                     int32_t* __restrict__ trace, int trace_cap) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int n_grp = d_in / group, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t j = blockIdx.x;
    const float top = (float)((1 << bits) - 1);
    // LDS carve-up
    double* v = reinterpret_cast<double*>(smem);                          // [d_in]
    double* quad = v + d_in;                                              // [n_grp][n_gamma]
    double* red_s = quad + n_grp * n_gamma;                               // [4]
    float* w = reinterpret_cast<float*>(red_s + 4);                       // [d_in]
    float* e = w + d_in;                                                  // [d_in]
    float* a_tab = e + d_in;                                              // [n_grp][n_gamma]
    float* enew = a_tab + n_grp * n_gamma;                                // [n_gamma][group]
    float* lo = enew + n_gamma * group;                                   // [n_grp]
    float* hi = lo + n_grp;                                               // [n_grp]
    int* cur = reinterpret_cast<int*>(hi + n_grp);                        // [n_grp]
    int* red_p = cur + n_grp;                                             // [4]

    const float* wj = Wt + j * (int64_t)d_in;
    for (int m = tid; m < d_in; m += 256) w[m] = wj[m];
    __syncthreads();
    for (int i = wave; i < n_grp; i += 4) {            // min / max per group
        float l = INFINITY, h = -INFINITY;
        for (int m = lane; m < group; m += 64) { const float x = w[i * group + m]; l = fminf(l, x); h = fmaxf(h, x); }
        for (int o = 32; o; o >>= 1) { l = fminf(l, __shfl_xor(l, o)); h = fmaxf(h, __shfl_xor(h, o)); }
        if (lane == 0) { lo[i] = l; hi[i] = h; cur[i] = n_gamma; }
    }
    __syncthreads();
    for (int p = tid; p < n_grp * n_gamma; p += 256) a_tab[p] = owc_scale(lo[p / n_gamma], hi[p / n_gamma], p % n_gamma + 1, n_gamma, top);
    __syncthreads();
    for (int m = tid; m < d_in; m += 256) e[m] = owc_resid(w[m], lo[m / group], a_tab[(m / group) * n_gamma + n_gamma - 1], top);
    __syncthreads();
    for (int r = tid; r < d_in; r += 256) {            // v = 2 H e  (H symmetric: walk down column r, coalesced)
        double acc = 0.0;
        for (int m = 0; m < d_in; ++m) acc += (double)H[(int64_t)m * d_in + r] * (double)e[m];
        v[r] = 2.0 * acc;
    }

    // quad(i, k) for all k of one group: Y = D H_ii accumulated per thread for one column c of H_ii
    auto quad_group = [&](int i) {
        __syncthreads();
        for (int p = tid; p < n_gamma * group; p += 256) {
            const int k = p / group, m = p % group;
            enew[p] = owc_resid(w[i * group + m], lo[i], a_tab[i * n_gamma + k], top);
        }
        for (int k = tid; k < n_gamma; k += 256) quad[i * n_gamma + k] = 0.0;
        __syncthreads();
        // each wavefront takes grid points k = wave, wave+4, ...; lanes stride over the columns c
        for (int k = wave; k < n_gamma; k += 4) {
            double part = 0.0;
            for (int c = lane; c < group; c += 64) {
                double y = 0.0;
                const float* hcol = H + (int64_t)(i * group) * d_in + i * group + c;     // H_ii[m][c], m down the rows
                for (int m = 0; m < group; ++m)
                    y += (double)hcol[(int64_t)m * d_in] * ((double)enew[k * group + m] - (double)e[i * group + m]);
                part += y * ((double)enew[k * group + c] - (double)e[i * group + c]);
            }
            for (int o = 32; o; o >>= 1) part += __shfl_xor(part, o);
            if (lane == 0) quad[i * n_gamma + k] = part;
        }
        __syncthreads();
    };
    for (int i = 0; i < n_grp; ++i) quad_group(i);

    int moves = 0;
    for (int t = 0; t < T; ++t) {
        // ---- scores and arg-min over (group, grid point)
        OwcBest best = {0.0, 0x7fffffff};
        for (int p = tid; p < n_grp * n_gamma; p += 256) {
            const int i = p / n_gamma, k = p % n_gamma;
            if (k + 1 == cur[i]) continue;
            const float a = a_tab[p], l = lo[i];
            double lin = 0.0;
            for (int m = 0; m < group; ++m) {
                const int c = i * group + m;
                lin += v[c] * ((double)owc_resid(w[c], l, a, top) - (double)e[c]);
            }
            const double s = quad[p] + lin;
            if (s < best.s) { best.s = s; best.p = p; }       // p ascends per thread: ties keep the smaller index
        }
        for (int o = 32; o; o >>= 1) {
            OwcBest other;
            other.s = __shfl_xor(best.s, o);
            other.p = __shfl_xor(best.p, o);
            best = owc_min(best, other);
        }
        if (lane == 0) { red_s[wave] = best.s; red_p[wave] = best.p; }
        __syncthreads();
        best.s = red_s[0]; best.p = red_p[0];
        for (int q = 1; q < 4; ++q) { OwcBest o2 = {red_s[q], red_p[q]}; best = owc_min(best, o2); }
        if (!(best.s < 0.0)) break;                            // no group can lower the loss
        const int is = best.p / n_gamma, ks = best.p % n_gamma;
        // ---- commit: v += 2 H[:, group] d, e <- e(i*, k*), quad(i*, .) recomputed
        __syncthreads();
        for (int m = tid; m < group; m += 256)                 // stage d* in enew[0..group)
            enew[m] = owc_resid(w[is * group + m], lo[is], a_tab[is * n_gamma + ks], top);
        __syncthreads();
        for (int r = tid; r < d_in; r += 256) {
            double acc = 0.0;
            const float* hcol = H + (int64_t)(is * group) * d_in + r;          // H[g0+m][r] = H[r][g0+m]
            for (int m = 0; m < group; ++m) acc += (double)hcol[(int64_t)m * d_in] * ((double)enew[m] - (double)e[is * group + m]);
            v[r] += 2.0 * acc;
        }
        __syncthreads();
        for (int m = tid; m < group; m += 256) e[is * group + m] = enew[m];
        if (tid == 0) {
            cur[is] = ks + 1;
            if (trace != nullptr && moves < trace_cap) trace[j * trace_cap + moves] = is * 4096 + ks + 1;
        }
        ++moves;
        quad_group(is);
    }
    __syncthreads();
    // ---- outputs: grid and codes of the chosen clipping strengths
    for (int i = tid; i < n_grp; i += 256) {
        scale[j * n_grp + i] = a_tab[i * n_gamma + cur[i] - 1];
        zero[j * n_grp + i] = lo[i];
        if (gamma_idx != nullptr) gamma_idx[j * n_grp + i] = cur[i];
    }
    for (int m = tid; m < d_in; m += 256) {
        const int i = m / group;
        Q[j * (int64_t)d_in + m] = (uint8_t)owc_code(w[m], lo[i], a_tab[i * n_gamma + cur[i] - 1], top);
    }
    if (tid == 0 && moves_out != nullptr) moves_out[j] = moves;
}

size_t owc_cd_lds_bytes(int64_t d_in, int64_t group, int n_gamma) {
    const int64_t n_grp = d_in / group;
    size_t b = 0;
    b += sizeof(double) * (d_in + n_grp * n_gamma + 4);
    b += sizeof(float) * (2 * d_in + n_grp * n_gamma + (int64_t)n_gamma * group + 2 * n_grp);
    b += sizeof(int) * (n_grp + 4);
    return cdq_align_up(b, 16);
}

}  // namespace

int owc_cd_launch(const float* H, const float* Wt, int64_t d_out, int64_t d_in, int bits, int64_t group, int n_gamma, int64_t T,
                  float* scale, float* zero, uint8_t* Q, int32_t* gamma_idx, int32_t* moves, int32_t* trace, int64_t trace_cap,
                  hipStream_t st) {
    if (d_out == 0) return CDQ_OK;
    const size_t lds = owc_cd_lds_bytes(d_in, group, n_gamma);
    if (lds > 160 * 1024 || d_in > (1 << 20) || d_out > 0x7fffffffLL || n_gamma > 4095) return CDQ_EUNSUPPORTED;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(owc_cd_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return CDQ_EHIP;
    hipLaunchKernelGGL(owc_cd_kernel, dim3((unsigned)d_out), dim3(256), lds, st, H, Wt, (int)d_in, bits, (int)group, n_gamma,
                       (int)(T > 0x7fffffffLL ? 0x7fffffffLL : T), scale, zero, Q, gamma_idx, moves, trace,
                       (int)(trace_cap > 0x7fffffffLL ? 0x7fffffffLL : trace_cap));
    CDQ_LAUNCH_CHECK();
    return CDQ_OK;
}

}  // namespace cdq
