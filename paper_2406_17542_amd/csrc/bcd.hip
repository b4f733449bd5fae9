// Block coordinate descent with random blocks of two coordinates (paper Algorithm 2; Algorithm 5
// for groups), weight-space form.  One workgroup owns a column for all T iterations; 2g, the codes,
// the Hessian diagonal and u = |2g| / (H_ii a_i) sit in LDS.  The loss change of moving the pair
// (i,k) to the levels (r_i, r_k) is
//     delta_i = a_i (r_i - q_i),   s_i = delta_i * fma(delta_i, H_ii, 2 g_i)      (same for k)
//     s(r_i, r_k) = fma(delta_i * delta_k, 2 H_ik, s_i + s_k).
// What depends only on the partition -- the pair (i,k), 2 H_ik, and the pair's threshold on u (below)
// -- is gathered once for all columns before the loop.  Per iteration:
//   1. every thread tests its pairs: a pair whose two u are under the threshold provably holds no
//      move with a negative score and is dropped; the others are counted, the first 16 queued;
//   2. few survivors (the usual case near a coordinate-wise optimum, the start the paper uses): the
//      level pairs of a survivor are spread over the lanes of a wavefront; many survivors: every
//      thread scores its own pairs over all level pairs;
//   3. the workgroup takes the minimum of (ordered score, pair, r_i, r_k): ties go to the first
//      pair of the partition, then the smaller r_i, then r_k;
//   4. if negative: 2g <- fma(2 delta_i, H[i,:], 2g), then the same with k; u refreshed; codes replaced.
// The entries of the next iteration are loaded while the current one is processed.
#include "cdq_internal.h"
#include "wave_min.h"

namespace cdq {
namespace {

constexpr int BCD_PPT = 4;          // pairs per thread at most

// A pair can be left out of the scoring when no move of it can have a negative score.  With
// rho = |H_ik| / sqrt(H_ii H_kk):  2 H_ik di dk >= -rho (H_ii di^2 + H_kk dk^2), so
//   s >= (1-rho)(H_ii di^2 + H_kk dk^2) - |2 g_i| |di| - |2 g_k| |dk|,
// and a nonzero step is at least one grid step a, so |2 g| |d| <= (|2 g| / a) d^2.  If
// u_i = |2 g_i| / (H_ii a_i) <= 1 - rho - tau and the same for k, every move has
// s >= tau (H_ii di^2 + H_kk dk^2) > 0 in exact arithmetic; the fp32 evaluation differs from that by
// a few 1e-7 of the same magnitude, far inside tau = 2^-10.  thr = 1 - rho - tau per pair; -1 (never
// dropped) when a diagonal entry is not positive.
constexpr float kBcdTau = 1.0f / 1024.0f;

__global__ __launch_bounds__(256) void bcd_pair_gather_kernel(const float* __restrict__ H, const int32_t* __restrict__ parts,
                                                              const int32_t* __restrict__ bad, int64_t d_in, int64_t n_items,
                                                              int2* __restrict__ pair_rec, float* __restrict__ pair_h2) {
    const int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x;        // x = t * (d_in/2) + p
    if (x >= n_items || *bad != 0) return;                            // indices are only followed once the check accepted them
    const int32_t i = parts[2 * x], k = parts[2 * x + 1];
    const float h2 = 2.0f * H[(int64_t)i * d_in + k];
    const float hii = H[(int64_t)i * d_in + i], hkk = H[(int64_t)k * d_in + k];
    float thr = -1.0f;
    if (hii > 0.0f && hkk > 0.0f) thr = 1.0f - (0.5f * fabsf(h2) * __frsqrt_rn(hii)) * __frsqrt_rn(hkk) - kBcdTau;
    pair_rec[x] = make_int2(i | (k << 16), __float_as_int(thr));
    pair_h2[x] = h2;
}

__global__ void bcd_fill_i32_kernel(int32_t* __restrict__ p, int64_t n, int32_t v) {
    const int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (x < n) p[x] = v;
}

// every entry of parts in range, every row a permutation (each value hit exactly once)
__global__ __launch_bounds__(256) void bcd_check_parts_kernel(const int32_t* __restrict__ parts, int d_in, int32_t* __restrict__ bad) {
    extern __shared__ int32_t seen[];
    const int32_t* row = parts + (int64_t)blockIdx.x * d_in;
    for (int c = threadIdx.x; c < d_in; c += 256) seen[c] = 0;
    __syncthreads();
    for (int c = threadIdx.x; c < d_in; c += 256) {
        const int32_t v = row[c];
        if (v < 0 || v >= d_in) atomicAdd(bad, 1);
        else if (atomicAdd(&seen[v], 1) != 0) atomicAdd(bad, 1);
    }
}

constexpr int BCD_FASTQ = 16;       // survivors up to this many are scored with the lanes spread over the level pairs

template <int BITS>
__global__ __launch_bounds__(1024) void bcd2_kernel(const float* __restrict__ H, const float* __restrict__ hdiag,
                                                    const float* __restrict__ G0, const float* __restrict__ scale,
                                                    uint8_t* __restrict__ Q, const int2* __restrict__ pair_rec,
                                                    const float* __restrict__ pair_h2, const int32_t* __restrict__ bad_parts,
                                                    int d_in, int group, int T, int score_all, int32_t* __restrict__ moves_out,
                                                    float* __restrict__ G_out, int32_t* __restrict__ trace, int trace_cap) {
    constexpr int L = 1 << BITS, C = L * L;
    constexpr int LP = C < 64 ? C : 64;          // lanes per survivor, survivors per wavefront pass, level pairs per lane
    constexpr int PPW = 64 / LP, CPL = C / LP;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63, wave = tid >> 6, n_waves = nt >> 6;
    const int n_grp = d_in / group, n_pairs = d_in / 2;
    const int64_t j = blockIdx.x;
    float* g2 = reinterpret_cast<float*>(smem);                  // [d_in]  2 g
    float* hd = g2 + d_in;                                       // [d_in]  H_ii
    float* u = hd + d_in;                                        // [d_in]  |2 g_i| / (H_ii a_i)
    int4* fastq = reinterpret_cast<int4*>(u + d_in);             // [BCD_FASTQ] p, i, k, bits of 2 H_ik
    uint64_t* slots = reinterpret_cast<uint64_t*>(fastq + BCD_FASTQ);        // [2][16] per-wavefront minima
    float* commit = reinterpret_cast<float*>(slots + 32);        // [2][4]: i, k (as int bits), 2 delta_i, 2 delta_k
    int* q_count = reinterpret_cast<int*>(commit + 8);           // [4] ring of survivor counters
    float* a = reinterpret_cast<float*>(q_count + 4);            // [n_grp]
    uint8_t* q = reinterpret_cast<uint8_t*>(a + n_grp);          // [d_in]

    if (*bad_parts != 0) {                                       // invalid partitions: leave the column untouched
        if (tid == 0 && moves_out != nullptr) moves_out[j] = -1;
        return;
    }
    for (int i = tid; i < n_grp; i += nt) a[i] = scale[j * n_grp + i];
    if (tid < 4) q_count[tid] = 0;
    __syncthreads();
    for (int c = tid; c < d_in; c += nt) {
        const float g = 2.0f * G0[j * (int64_t)d_in + c], h = hdiag[c];
        g2[c] = g;
        hd[c] = h;
        u[c] = __fdiv_rn(fabsf(g), h * a[c / group]);
        q[c] = Q[j * (int64_t)d_in + c];
    }

    // entries of the next iteration are in flight while the current one is processed
    int2 nxt_rec[BCD_PPT];
    float nxt_h2[BCD_PPT];
    auto fetch = [&](int t) {
#pragma unroll
        for (int pp = 0; pp < BCD_PPT; ++pp) {
            const int p = tid + pp * nt;
            if (p < n_pairs && t < T) {
                nxt_rec[pp] = pair_rec[(int64_t)t * n_pairs + p];
                nxt_h2[pp] = pair_h2[(int64_t)t * n_pairs + p];
            }
        }
    };
    fetch(0);
    __syncthreads();

    int moves = 0;
    for (int t = 0; t < T; ++t) {
        int* cnt = q_count + (t & 3);
        int2 rec[BCD_PPT];
        float h2[BCD_PPT];
        bool need[BCD_PPT];
        // ---- which pairs need scoring (all loads first, no short-circuit: one pass of straight-line code)
        float ui[BCD_PPT], uk[BCD_PPT];
#pragma unroll
        for (int pp = 0; pp < BCD_PPT; ++pp) {
            rec[pp] = nxt_rec[pp]; h2[pp] = nxt_h2[pp];
            const bool valid = tid + pp * nt < n_pairs;
            ui[pp] = u[valid ? (rec[pp].x & 0xffff) : 0];
            uk[pp] = u[valid ? (int)((uint32_t)rec[pp].x >> 16) : 0];
        }
        bool any = false;
#pragma unroll
        for (int pp = 0; pp < BCD_PPT; ++pp) {
            const float thr = __int_as_float(rec[pp].y);
            const bool quiet = (ui[pp] <= thr) & (uk[pp] <= thr);             // NaN keeps the pair
            need[pp] = (tid + pp * nt < n_pairs) & ((score_all != 0) | !quiet);
            any |= need[pp];
        }
        if (__ballot(any)) {
#pragma unroll
            for (int pp = 0; pp < BCD_PPT; ++pp) {
                const unsigned long long m = __ballot(need[pp]);
                if (m) {
                    const int first = __builtin_ctzll(m);
                    int base = 0;
                    if (lane == first) base = atomicAdd(cnt, __builtin_popcountll(m));
                    base = __builtin_amdgcn_readlane(base, first);
                    const int pos = base + __builtin_popcountll(m & ((1ull << lane) - 1ull));
                    if (need[pp] && pos < BCD_FASTQ)
                        fastq[pos] = make_int4(tid + pp * nt, rec[pp].x & 0xffff, (int)((uint32_t)rec[pp].x >> 16), __float_as_int(h2[pp]));
                }
            }
        }
        fetch(t + 1);
        __syncthreads();
        const int n_q = *cnt;
        if (tid == 0) q_count[(t + 2) & 3] = 0;       // two ahead: its next use is after the next iteration's barrier
        if (n_q == 0) continue;

        float best_s = 0.0f, best_di = 0.0f, best_dk = 0.0f;
        uint32_t best_pay = 0xffffffffu;
        int best_i = 0, best_k = 0;
        if (n_q <= BCD_FASTQ) {
            // ---- few survivors: LP lanes share one pair, each lane scores CPL level pairs
            const int sub = lane % LP;
            for (int x = wave * PPW + lane / LP; x < n_q; x += n_waves * PPW) {
                const int4 e = fastq[x];
                const int i = e.y, k = e.z;
                const float ai = a[i / group], ak = a[k / group], gi = g2[i], gk = g2[k], hii = hd[i], hkk = hd[k];
                const float hh = __int_as_float(e.w);
                const int qi = q[i], qk = q[k];
#pragma unroll
                for (int m = 0; m < CPL; ++m) {
                    const int c = sub + m * LP, ri = c >> BITS, rk = c & (L - 1);
                    const float di = ai * (float)(ri - qi), dk = ak * (float)(rk - qk);
                    const float si = di * fmaf(di, hii, gi), sk = dk * fmaf(dk, hkk, gk);
                    const float s = fmaf(di * dk, hh, si + sk);
                    const uint32_t pay = ((uint32_t)e.x << 8) | (uint32_t)(ri << 4) | (uint32_t)rk;
                    if (s < best_s || (s == best_s && s < 0.0f && pay < best_pay)) {
                        best_s = s; best_pay = pay; best_di = di; best_dk = dk; best_i = i; best_k = k;
                    }
                }
            }
        } else {
            // ---- many survivors: every thread scores its own pairs over all level pairs
#pragma unroll
            for (int pp = 0; pp < BCD_PPT; ++pp) {
                if (need[pp]) {
                    const int p = tid + pp * nt;
                    const int i = rec[pp].x & 0xffff, k = (int)((uint32_t)rec[pp].x >> 16);
                    const float ai = a[i / group], ak = a[k / group], gi = g2[i], gk = g2[k], hii = hd[i], hkk = hd[k];
                    const int qi = q[i], qk = q[k];
                    float dk[L], sk[L];
#pragma unroll
                    for (int r = 0; r < L; ++r) {
                        dk[r] = ak * (float)(r - qk);
                        sk[r] = dk[r] * fmaf(dk[r], hkk, gk);
                    }
                    float pmin = 0.0f;               // first a pass that only keeps the minimum ...
#pragma unroll
                    for (int ri = 0; ri < L; ++ri) {
                        const float di = ai * (float)(ri - qi);
                        const float si = di * fmaf(di, hii, gi);
#pragma unroll
                        for (int rk = 0; rk < L; ++rk) pmin = fminf(pmin, fmaf(di * dk[rk], h2[pp], si + sk[rk]));
                    }
                    if (pmin < best_s) {             // ... and, for a pair that beats the thread's best, one that finds where
                        float cur = 0.0f;
#pragma unroll
                        for (int ri = 0; ri < L; ++ri) {
                            const float di = ai * (float)(ri - qi);
                            const float si = di * fmaf(di, hii, gi);
#pragma unroll
                            for (int rk = 0; rk < L; ++rk) {
                                const float s = fmaf(di * dk[rk], h2[pp], si + sk[rk]);
                                if (s < cur) {
                                    cur = s; best_di = di; best_dk = dk[rk];
                                    best_pay = ((uint32_t)p << 8) | (uint32_t)(ri << 4) | (uint32_t)rk;
                                }
                            }
                        }
                        best_s = cur; best_i = i; best_k = k;
                    }
                }
            }
        }
        // ---- workgroup minimum of (ordered score, pair, levels)
        const uint64_t wkey = wave_min_key(order_bits(best_s), best_pay);
        uint64_t* slot = slots + (t & 1) * 16;
        if (lane == 0) slot[wave] = wkey;
        __syncthreads();
        uint64_t key = slot[0];
        for (int w = 1; w < n_waves; ++w) key = umin64(key, slot[w]);
        if ((uint32_t)(key >> 32) >= kOrderedZero) continue;          // no pair lowers the loss under this partition
        float* cm = commit + (t & 1) * 4;
        if (best_pay == (uint32_t)key && order_bits(best_s) == (uint32_t)(key >> 32)) {      // exactly one thread
            cm[0] = __int_as_float(best_i); cm[1] = __int_as_float(best_k);
            cm[2] = 2.0f * best_di; cm[3] = 2.0f * best_dk;
            q[best_i] = (uint8_t)((best_pay >> 4) & 15u);
            q[best_k] = (uint8_t)(best_pay & 15u);
            if (trace != nullptr && moves < trace_cap) {
                int32_t* tr = trace + (j * trace_cap + moves) * 4;
                tr[0] = t; tr[1] = (int32_t)(best_pay >> 8);
                tr[2] = (int32_t)(((best_pay >> 4) & 15u) | ((best_pay & 15u) << 4));
                tr[3] = __float_as_int(best_s);
            }
        }
        ++moves;
        __syncthreads();
        const int ci = __float_as_int(cm[0]), ck = __float_as_int(cm[1]);
        const float tdi = cm[2], tdk = cm[3];
        const float* hi = H + (int64_t)ci * d_in;
        const float* hk = H + (int64_t)ck * d_in;
        for (int c = 4 * tid; c < d_in; c += 4 * nt) {
            const float4 x = *reinterpret_cast<const float4*>(hi + c);
            const float4 y = *reinterpret_cast<const float4*>(hk + c);
            float4 g = *reinterpret_cast<float4*>(g2 + c);
            const float4 h = *reinterpret_cast<const float4*>(hd + c);
            g.x = fmaf(tdk, y.x, fmaf(tdi, x.x, g.x));
            g.y = fmaf(tdk, y.y, fmaf(tdi, x.y, g.y));
            g.z = fmaf(tdk, y.z, fmaf(tdi, x.z, g.z));
            g.w = fmaf(tdk, y.w, fmaf(tdi, x.w, g.w));
            *reinterpret_cast<float4*>(g2 + c) = g;
            float4 un;
            un.x = __fdiv_rn(fabsf(g.x), h.x * a[c / group]);
            un.y = __fdiv_rn(fabsf(g.y), h.y * a[(c + 1) / group]);
            un.z = __fdiv_rn(fabsf(g.z), h.z * a[(c + 2) / group]);
            un.w = __fdiv_rn(fabsf(g.w), h.w * a[(c + 3) / group]);
            *reinterpret_cast<float4*>(u + c) = un;
        }
        __syncthreads();
    }
    __syncthreads();
    for (int c = tid; c < d_in; c += nt) {
        Q[j * (int64_t)d_in + c] = q[c];
        if (G_out != nullptr) G_out[j * (int64_t)d_in + c] = 0.5f * g2[c];
    }
    if (tid == 0 && moves_out != nullptr) moves_out[j] = moves;
}

size_t bcd_lds_bytes(int64_t d_in, int64_t group) {
    const int64_t n_grp = d_in / group;
    return cdq_align_up(sizeof(float) * 3 * d_in + 16 * BCD_FASTQ + sizeof(uint64_t) * 32 + sizeof(float) * 8 + sizeof(int) * 4 +
                        sizeof(float) * n_grp + (size_t)d_in, 16);
}

}  // namespace

// workspace: G0 [d_out][d_in] fp32 | hdiag [d_in] | pair_rec [T][d_in/2] int2 | pair_h2 [T][d_in/2] | flag
size_t bcd_workspace_bytes(int64_t d_out, int64_t d_in, int64_t T) {
    return cdq_align_up((size_t)d_out * d_in * sizeof(float), 256) + cdq_align_up((size_t)d_in * sizeof(float), 256) +
           cdq_align_up((size_t)T * (d_in / 2) * sizeof(int2), 256) + cdq_align_up((size_t)T * (d_in / 2) * sizeof(float), 256) + 256;
}

int bcd_launch(const float* H, const float* Wt, const float* scale, const float* zero, uint8_t* Q, int64_t d_out, int64_t d_in,
               int bits, int64_t group, const int32_t* parts, int64_t T, int32_t* moves, float* G_out, int32_t* trace,
               int64_t trace_cap, bool score_all, void* ws, size_t ws_bytes, hipStream_t st) {
    if (d_out == 0 || T == 0) {
        if (T == 0 && d_out > 0 && moves != nullptr) {
            hipLaunchKernelGGL(bcd_fill_i32_kernel, dim3((unsigned)((d_out + 255) / 256)), dim3(256), 0, st, moves, d_out, 0);
            CDQ_LAUNCH_CHECK();
        }
        if (T == 0 && d_out > 0 && G_out != nullptr) return gradient_launch(H, Wt, scale, zero, Q, d_out, d_in, group, G_out, st);
        return CDQ_OK;
    }
    int nt = 256;
    while ((int64_t)nt * BCD_PPT < d_in / 2) nt *= 2;
    const size_t lds = bcd_lds_bytes(d_in, group);
    if (nt > 1024 || lds > 160 * 1024 || d_in % 4 != 0 || ((uintptr_t)H & 15) || d_in >= (1 << 24) || T > 0x7fffffffLL || d_out > 0x7fffffffLL) return CDQ_EUNSUPPORTED;
    if (ws == nullptr || ((uintptr_t)ws & 255) || ws_bytes < bcd_workspace_bytes(d_out, d_in, T)) return CDQ_EWORKSPACE;
    char* wp = (char*)ws;
    float* G0 = (float*)wp;           wp += cdq_align_up((size_t)d_out * d_in * sizeof(float), 256);
    float* hdiag = (float*)wp;        wp += cdq_align_up((size_t)d_in * sizeof(float), 256);
    int2* pair_rec = (int2*)wp;       wp += cdq_align_up((size_t)T * (d_in / 2) * sizeof(int2), 256);
    float* pair_h2 = (float*)wp;      wp += cdq_align_up((size_t)T * (d_in / 2) * sizeof(float), 256);
    int32_t* bad = (int32_t*)wp;

    hipLaunchKernelGGL(bcd_fill_i32_kernel, dim3(1), dim3(64), 0, st, bad, (int64_t)1, 0);
    CDQ_LAUNCH_CHECK();
    hipLaunchKernelGGL(bcd_check_parts_kernel, dim3((unsigned)T), dim3(256), sizeof(int32_t) * (size_t)d_in, st, parts, (int)d_in, bad);
    CDQ_LAUNCH_CHECK();
    int rc = gradient_launch(H, Wt, scale, zero, Q, d_out, d_in, group, G0, st);
    if (rc != CDQ_OK) return rc;
    rc = extract_diag_launch(H, d_in, hdiag, st);
    if (rc != CDQ_OK) return rc;
    const int64_t n_items = T * (d_in / 2);
    hipLaunchKernelGGL(bcd_pair_gather_kernel, dim3((unsigned)((n_items + 255) / 256)), dim3(256), 0, st, H, parts,
                       (const int32_t*)bad, d_in, n_items, pair_rec, pair_h2);
    CDQ_LAUNCH_CHECK();
#define BCD_CASE(B)                                                                                                              \
    case B:                                                                                                                      \
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(bcd2_kernel<B>), hipFuncAttributeMaxDynamicSharedMemorySize,       \
                                (int)lds) != hipSuccess)                                                                         \
            return CDQ_EHIP;                                                                                                     \
        hipLaunchKernelGGL((bcd2_kernel<B>), dim3((unsigned)d_out), dim3(nt), lds, st, H, (const float*)hdiag, (const float*)G0, \
                           scale, Q, (const int2*)pair_rec, (const float*)pair_h2, (const int32_t*)bad, (int)d_in, (int)group, (int)T, score_all ? 1 : 0, moves, \
                           G_out, trace, (int)(trace_cap > 0x7fffffffLL ? 0x7fffffffLL : trace_cap));                            \
        break;
    switch (bits) {
        BCD_CASE(2) BCD_CASE(3) BCD_CASE(4)
        default: return CDQ_EINVAL;
    }
#undef BCD_CASE
    CDQ_LAUNCH_CHECK();
    return CDQ_OK;
}

}  // namespace cdq
