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


// ------------------------------------------------------------------------------------------------
// Tiled kernel for group % 4 == 0.  Algebra: with e_c the current residual of group i and
// e_k the residual for grid point k,
//   score(i,k) = d^T H_ii d + v_i^T d,  d = e_k - e_c
//              = F(i,k) - F(i,cur_i),   F(i,k) = A(i,k) + sum_m e_k[m] z[m],
//   A(i,k) = e_k^T H_ii e_k             (depends on nothing that moves: computed once),
//   z      = v - 2 blockdiag(H) e       (the part of 2He that comes from the other groups).
// A move of group i* by d* changes z only outside that group: z[c] += 2 sum_m H[g0*+m][c] d*[m].
// So an iteration is: F for every (group, grid point), arg-min, one rank-`group` update of z.
// v = 2He of the MinMax start comes from the fp64 GEMM (G64 = He); the block-diagonal part is
// taken off here.
constexpr int ONT = 512;      // threads per column
constexpr int KT = 7;         // grid points per wavefront in the A pass
constexpr int LPP = 8;        // lanes per (group, grid point) pair in the F pass

// Residual for one weight with the division replaced by a multiplication with r = 1/a; exact because
// the quotient is redone with a true division whenever it lies close enough to a rounding boundary
// for the two to disagree (|t_mul - t_div| <= 1.5 * 2^-23 * t, the window is 2^-20 * t).
__device__ __forceinline__ float owc_resid_fast(float x, float lo, float a, float r, float top) {
    const float y = x - lo;
    const float t = y * r;
    float q = rintf(t);
    if (__builtin_expect(!(fabsf(t - q) < 0.5f - t * 0x1p-20f), 0)) q = rintf(__fdiv_rn(y, a));
    q = fminf(fmaxf(q, 0.0f), top);
    return fmaf(a, q, lo) - x;
}

__global__ __launch_bounds__(ONT) __attribute__((amdgpu_waves_per_eu(4, 4))) void owc_cd_tiled_kernel(const float* __restrict__ H, const float* __restrict__ Wt,
                                                           const double* __restrict__ G64, int d_in, int bits, int group,
                                                           int n_gamma, int T, float* __restrict__ scale, float* __restrict__ zero,
                                                           uint8_t* __restrict__ Q, int32_t* __restrict__ gamma_idx,
                                                           int32_t* __restrict__ moves_out, int32_t* __restrict__ trace,
                                                           int trace_cap, int region_bytes) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int n_grp = d_in / group, n_pairs = n_grp * n_gamma;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t j = blockIdx.x;
    const float top = (float)((1 << bits) - 1);
    // LDS: [region: E staging during the A pass | z, F, dstar afterwards] A red_s | w e a_tab r_tab lo hi | cur red_p
    float* E = reinterpret_cast<float*>(smem);                            // [n_gamma][group]
    double* z = reinterpret_cast<double*>(smem);                          // [d_in]
    double* F = z + d_in;                                                 // [n_pairs]
    double* dstar = F + n_pairs;                                          // [group]
    double* A = reinterpret_cast<double*>(smem + region_bytes);           // [n_pairs]
    double* red_s = A + n_pairs;                                          // [8]
    float* w = reinterpret_cast<float*>(red_s + 8);                       // [d_in]
    float* e = w + d_in;                                                  // [d_in]
    float* a_tab = e + d_in;                                              // [n_pairs]
    float* r_tab = a_tab + n_pairs;                                       // [n_pairs]
    float* lo = r_tab + n_pairs;                                          // [n_grp]
    float* hi = lo + n_grp;                                               // [n_grp]
    int* cur = reinterpret_cast<int*>(hi + n_grp);                        // [n_grp]
    int* red_p = cur + n_grp;                                             // [8]

    const float* wj = Wt + j * (int64_t)d_in;
    for (int m = 4 * tid; m < d_in; m += 4 * ONT) *reinterpret_cast<float4*>(w + m) = *reinterpret_cast<const float4*>(wj + m);
    __syncthreads();
    for (int i = wave; i < n_grp; i += ONT / 64) {
        float l = INFINITY, h = -INFINITY;
        for (int m = lane; m < group; m += 64) { const float x = w[i * group + m]; l = fminf(l, x); h = fmaxf(h, x); }
        for (int o = 32; o; o >>= 1) { l = fminf(l, __shfl_xor(l, o)); h = fmaxf(h, __shfl_xor(h, o)); }
        if (lane == 0) { lo[i] = l; hi[i] = h; cur[i] = n_gamma; }
    }
    __syncthreads();
    for (int p = tid; p < n_pairs; p += ONT) {
        const float a = owc_scale(lo[p / n_gamma], hi[p / n_gamma], p % n_gamma + 1, n_gamma, top);
        a_tab[p] = a;
        r_tab[p] = __fdiv_rn(1.0f, a);
    }
    __syncthreads();
    for (int m = tid; m < d_in; m += ONT) e[m] = owc_resid(w[m], lo[m / group], a_tab[(m / group) * n_gamma + n_gamma - 1], top);

    // ---- A pass: A(i,k) = e_k^T H_ii e_k.  A wavefront takes KT grid points; its lanes take a 4-column strip of
    // H_ii each, over one of MS slices of the rows, keep a KT x 4 block of (E H_ii) in registers, and finish with
    // the dot product against e_k and a butterfly sum.
    const int n_cb = group / 4;
    int MS = 1;
    while (MS * 2 * n_cb <= 64 && group % (MS * 2 * 4) == 0) MS *= 2;
    const int mlen = group / MS, n_items = n_cb * MS;
    for (int i = 0; i < n_grp; ++i) {
        const int g0 = i * group;
        __syncthreads();
        for (int p = tid; p < n_gamma * group; p += ONT) {
            const int k = p / group, m = p % group;
            E[p] = owc_resid(w[g0 + m], lo[i], a_tab[i * n_gamma + k], top);
        }
        __syncthreads();
        for (int kb = wave; kb * KT < n_gamma; kb += ONT / 64) {
            double s[KT];
            int krow[KT];
#pragma unroll
            for (int kk = 0; kk < KT; ++kk) { s[kk] = 0.0; krow[kk] = min(kb * KT + kk, n_gamma - 1) * group; }
            for (int it = lane; it < n_items; it += 64) {
                const int cb = it % n_cb, ms = it / n_cb;
                double acc[KT][4];
#pragma unroll
                for (int kk = 0; kk < KT; ++kk)
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc) acc[kk][cc] = 0.0;
                const float* hp = H + (int64_t)(g0 + ms * mlen) * d_in + g0 + 4 * cb;
                for (int m = ms * mlen; m < (ms + 1) * mlen; m += 4) {
                    float4 ev[KT];
#pragma unroll
                    for (int kk = 0; kk < KT; ++kk) ev[kk] = *reinterpret_cast<const float4*>(E + krow[kk] + m);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float4 h4 = *reinterpret_cast<const float4*>(hp + (int64_t)r * d_in);
                        const double hd[4] = {(double)h4.x, (double)h4.y, (double)h4.z, (double)h4.w};
#pragma unroll
                        for (int kk = 0; kk < KT; ++kk) {
                            const double ed = (double)(r == 0 ? ev[kk].x : r == 1 ? ev[kk].y : r == 2 ? ev[kk].z : ev[kk].w);
#pragma unroll
                            for (int cc = 0; cc < 4; ++cc) acc[kk][cc] = fma(ed, hd[cc], acc[kk][cc]);
                        }
                    }
                    hp += 4 * (int64_t)d_in;
                }
#pragma unroll
                for (int kk = 0; kk < KT; ++kk) {
                    const float4 ec = *reinterpret_cast<const float4*>(E + krow[kk] + 4 * cb);
                    s[kk] += (acc[kk][0] * (double)ec.x + acc[kk][1] * (double)ec.y) + (acc[kk][2] * (double)ec.z + acc[kk][3] * (double)ec.w);
                }
            }
#pragma unroll
            for (int kk = 0; kk < KT; ++kk) {
                double x = s[kk];
                for (int o = 32; o; o >>= 1) x += __shfl_xor(x, o);
                if (lane == 0 && kb * KT + kk < n_gamma) A[i * n_gamma + kb * KT + kk] = x;
            }
        }
    }
    __syncthreads();

    // ---- z = 2 (He - blockdiag(H) e) for the MinMax start
    for (int c = 4 * tid; c < d_in; c += 4 * ONT) {
        const int g0 = (c / group) * group;
        double acc[4] = {0.0, 0.0, 0.0, 0.0};
        const float* hp = H + (int64_t)g0 * d_in + c;
#pragma unroll 8
        for (int m = 0; m < group; ++m) {
            const float4 h4 = *reinterpret_cast<const float4*>(hp + (int64_t)m * d_in);
            const double x = (double)e[g0 + m];
            acc[0] = fma((double)h4.x, x, acc[0]); acc[1] = fma((double)h4.y, x, acc[1]);
            acc[2] = fma((double)h4.z, x, acc[2]); acc[3] = fma((double)h4.w, x, acc[3]);
        }
        const double* gp = G64 + j * (int64_t)d_in + c;
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) z[c + cc] = 2.0 * (gp[cc] - acc[cc]);
    }
    __syncthreads();

    int moves = 0;
    const int sub = tid % LPP, pslot = tid / LPP;
    for (int t = 0; t < T; ++t) {
        // ---- F(i,k) = A(i,k) + sum_m e_k[m] z[m]
        for (int p = pslot; p < n_pairs; p += ONT / LPP) {
            const int i = p / n_gamma, g0 = i * group;
            const float a = a_tab[p], r = r_tab[p], l = lo[i];
            double acc4[4] = {0.0, 0.0, 0.0, 0.0};
            for (int m = 4 * sub; m < group; m += 4 * LPP) {          // four consecutive weights per lane and step
                const float4 w4 = *reinterpret_cast<const float4*>(w + g0 + m);
                const double2 z01 = *reinterpret_cast<const double2*>(z + g0 + m), z23 = *reinterpret_cast<const double2*>(z + g0 + m + 2);
                acc4[0] = fma((double)owc_resid_fast(w4.x, l, a, r, top), z01.x, acc4[0]);
                acc4[1] = fma((double)owc_resid_fast(w4.y, l, a, r, top), z01.y, acc4[1]);
                acc4[2] = fma((double)owc_resid_fast(w4.z, l, a, r, top), z23.x, acc4[2]);
                acc4[3] = fma((double)owc_resid_fast(w4.w, l, a, r, top), z23.y, acc4[3]);
            }
            double acc = (acc4[0] + acc4[1]) + (acc4[2] + acc4[3]);
#pragma unroll
            for (int o = 1; o < LPP; o <<= 1) acc += __shfl_xor(acc, o);
            if (sub == 0) F[p] = A[p] + acc;
        }
        __syncthreads();
        // ---- arg-min of F(i,k) - F(i,cur_i); ties: smaller group, then smaller grid index
        OwcBest best = {0.0, 0x7fffffff};
        for (int p = tid; p < n_pairs; p += ONT) {
            const int i = p / n_gamma, k = p % n_gamma;
            if (k + 1 == cur[i]) continue;
            const double sc = F[p] - F[i * n_gamma + cur[i] - 1];
            if (sc < best.s) { best.s = sc; best.p = p; }
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
        for (int q = 1; q < ONT / 64; ++q) { OwcBest o2 = {red_s[q], red_p[q]}; best = owc_min(best, o2); }
        if (!(best.s < 0.0)) break;
        const int is = best.p / n_gamma, g0s = is * group;
        // ---- commit
        for (int m = tid; m < group; m += ONT) {
            const float en = owc_resid(w[g0s + m], lo[is], a_tab[best.p], top);
            dstar[m] = (double)en - (double)e[g0s + m];
            e[g0s + m] = en;
        }
        if (tid == 0) {
            cur[is] = best.p % n_gamma + 1;
            if (trace != nullptr && moves < trace_cap) trace[j * trace_cap + moves] = is * 4096 + best.p % n_gamma + 1;
        }
        ++moves;
        __syncthreads();
        for (int c = 4 * tid; c < d_in; c += 4 * ONT) {
            if (c / group == is) continue;
            double acc[4] = {0.0, 0.0, 0.0, 0.0};
            const float* hp = H + (int64_t)g0s * d_in + c;
#pragma unroll 8
            for (int m = 0; m < group; ++m) {
                const float4 h4 = *reinterpret_cast<const float4*>(hp + (int64_t)m * d_in);
                const double x = dstar[m];
                acc[0] = fma((double)h4.x, x, acc[0]); acc[1] = fma((double)h4.y, x, acc[1]);
                acc[2] = fma((double)h4.z, x, acc[2]); acc[3] = fma((double)h4.w, x, acc[3]);
            }
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) z[c + cc] += 2.0 * acc[cc];
        }
        __syncthreads();
    }
    __syncthreads();
    for (int i = tid; i < n_grp; i += ONT) {
        scale[j * n_grp + i] = a_tab[i * n_gamma + cur[i] - 1];
        zero[j * n_grp + i] = lo[i];
        if (gamma_idx != nullptr) gamma_idx[j * n_grp + i] = cur[i];
    }
    for (int m = tid; m < d_in; m += ONT) {
        const int i = m / group;
        Q[j * (int64_t)d_in + m] = (uint8_t)owc_code(w[m], lo[i], a_tab[i * n_gamma + cur[i] - 1], top);
    }
    if (tid == 0 && moves_out != nullptr) moves_out[j] = moves;
}

size_t owc_cd_tiled_region_bytes(int64_t d_in, int64_t group, int n_gamma) {
    const int64_t n_pairs = (d_in / group) * n_gamma;
    const size_t after = sizeof(double) * (d_in + n_pairs + group);
    const size_t staging = sizeof(float) * (size_t)n_gamma * group;
    return cdq_align_up(after > staging ? after : staging, 16);
}
size_t owc_cd_tiled_lds_bytes(int64_t d_in, int64_t group, int n_gamma) {
    const int64_t n_grp = d_in / group, n_pairs = n_grp * n_gamma;
    size_t b = owc_cd_tiled_region_bytes(d_in, group, n_gamma);
    b += sizeof(double) * (n_pairs + 8);
    b += sizeof(float) * (2 * d_in + 2 * n_pairs + 2 * n_grp);
    b += sizeof(int) * (n_grp + 8);
    return cdq_align_up(b, 16);
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

size_t owc_cd_workspace_bytes(int64_t d_out, int64_t d_in) {
    return cdq_align_up((size_t)d_out * (size_t)d_in * sizeof(double), 256);
}

int owc_cd_launch(const float* H, const float* Wt, int64_t d_out, int64_t d_in, int bits, int64_t group, int n_gamma, int64_t T,
                  float* scale, float* zero, uint8_t* Q, int32_t* gamma_idx, int32_t* moves, int32_t* trace, int64_t trace_cap,
                  void* ws, size_t ws_bytes, bool force_simple, hipStream_t st) {
    if (d_out == 0) return CDQ_OK;
    if (d_in > (1 << 20) || d_out > 0x7fffffffLL || n_gamma > 4095) return CDQ_EUNSUPPORTED;
    const int Ti = (int)(T > 0x7fffffffLL ? 0x7fffffffLL : T);
    const int cap = (int)(trace_cap > 0x7fffffffLL ? 0x7fffffffLL : trace_cap);
    const size_t lds_tiled = owc_cd_tiled_lds_bytes(d_in, group, n_gamma);
    const bool tiled = !force_simple && group % 4 == 0 && ((uintptr_t)H & 15) == 0 && ((uintptr_t)Wt & 15) == 0 && lds_tiled <= 160 * 1024;
    if (tiled) {
        if (ws == nullptr || ((uintptr_t)ws & 255) || ws_bytes < owc_cd_workspace_bytes(d_out, d_in)) return CDQ_EWORKSPACE;
        double* G64 = (double*)ws;
        // MinMax start (gamma = 1) into the output buffers, He of it by the fp64 GEMM
        int rc = rtn_launch(Wt, d_out, d_in, bits, group, scale, zero, Q, st);
        if (rc != CDQ_OK) return rc;
        rc = gradient_launch(H, Wt, scale, zero, Q, d_out, d_in, group, nullptr, st, G64);
        if (rc != CDQ_OK) return rc;
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(owc_cd_tiled_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds_tiled) != hipSuccess)
            return CDQ_EHIP;
        hipLaunchKernelGGL(owc_cd_tiled_kernel, dim3((unsigned)d_out), dim3(ONT), lds_tiled, st, H, Wt, (const double*)G64, (int)d_in,
                           bits, (int)group, n_gamma, Ti, scale, zero, Q, gamma_idx, moves, trace, cap,
                           (int)owc_cd_tiled_region_bytes(d_in, group, n_gamma));
        CDQ_LAUNCH_CHECK();
        return CDQ_OK;
    }
    const size_t lds = owc_cd_lds_bytes(d_in, group, n_gamma);
    if (lds > 160 * 1024) return CDQ_EUNSUPPORTED;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(owc_cd_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return CDQ_EHIP;
    hipLaunchKernelGGL(owc_cd_kernel, dim3((unsigned)d_out), dim3(256), lds, st, H, Wt, (int)d_in, bits, (int)group, n_gamma, Ti,
                       scale, zero, Q, gamma_idx, moves, trace, cap);
    CDQ_LAUNCH_CHECK();
    return CDQ_OK;
}

}  // namespace cdq
