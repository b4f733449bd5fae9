// Block coordinate descent with random blocks of two coordinates (paper Algorithm 2; Algorithm 5
// for groups), weight-space form.  Two kernels compute the same thing: bcd2_multi_kernel (further
// down) gives a workgroup several columns that share each row of the pair table and is used where
// their state fits in LDS; bcd2_kernel, described here, gives a workgroup one column for all T
// iterations; 2g, the codes, the Hessian diagonal and u = |2g| / (H_ii a_i) sit in LDS.  The loss change of moving the pair
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
#include <type_traits>

namespace cdq {
namespace {

constexpr int BCD_PPT = 4;          // pairs per thread at most

// A pair can be left out of the scoring when no move of it can have a negative score.  With
// rho = |H_ik| / sqrt(H_ii H_kk):  2 H_ik di dk >= -rho (H_ii di^2 + H_kk dk^2), so
//   s >= (1-rho)(H_ii di^2 + H_kk dk^2) - |2 g_i| |di| - |2 g_k| |dk|,
// and a nonzero step is at least one grid step a, so |2 g| |d| <= (|2 g| / a) d^2.  If
// u_i = |2 g_i| / (H_ii a_i) <= 1 - rho - tau and the same for k, every move has
// s >= tau (H_ii di^2 + H_kk dk^2) > 0 in exact arithmetic; the fp32 evaluation differs from that by
// less than 1e-6 of the same magnitude (five roundings of 2^-24 on terms that sum to at most three times it),
// far inside tau = 2^-14.  thr = 1 - rho - tau per pair; -1 (never dropped) when a diagonal entry is not
// positive.  A larger tau only costs time: coordinates with u within tau of 1 keep all their pairs alive.
constexpr float kBcdTau = 1.0f / 16384.0f;

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

// every entry of parts in range, every row a permutation (each value hit exactly once): one bit per value in LDS
__global__ __launch_bounds__(256) void bcd_check_parts_kernel(const int32_t* __restrict__ parts, int d_in, int32_t* __restrict__ bad) {
    extern __shared__ uint32_t seen[];
    const int32_t* row = parts + (int64_t)blockIdx.x * d_in;
    for (int c = threadIdx.x; c < (d_in + 31) / 32; c += 256) seen[c] = 0;
    __syncthreads();
    for (int c = threadIdx.x; c < d_in; c += 256) {
        const int32_t v = row[c];
        if (v < 0 || v >= d_in) atomicAdd(bad, 1);
        else if (atomicOr(&seen[v >> 5], 1u << (v & 31)) & (1u << (v & 31))) atomicAdd(bad, 1);
    }
}

constexpr int BCD_FASTQ = 16;       // survivors up to this many are scored with the lanes spread over the level pairs

// A coordinate at an end of its grid whose gradient asks for a step past that end cannot lower the loss on its own: every
// move it still has, delta = a (r - q), satisfies delta * 2g >= 0, so delta (delta H_ii + 2g) >= delta^2 H_ii, and the pair
// bound holds with u = 0 for it.  (A non-positive step size says nothing about directions: then the plain u is used.)
__device__ __forceinline__ bool bcd_blocked(float g2, float a, int q, int top) {
    return (a > 0.0f) & (((g2 > 0.0f) & (q == 0)) | ((g2 < 0.0f) & (q == top)));
}

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
        const uint8_t qc = Q[j * (int64_t)d_in + c];
        const float ac = a[c / group];
        u[c] = bcd_blocked(g, ac, qc, L - 1) ? 0.0f : __fdiv_rn(fabsf(g), h * ac);
        q[c] = qc;
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
            const uchar4 qv = *reinterpret_cast<const uchar4*>(q + c);              // the codes after this move
            const float a0 = a[c / group], a1 = a[(c + 1) / group], a2 = a[(c + 2) / group], a3 = a[(c + 3) / group];
            float4 un;
            un.x = bcd_blocked(g.x, a0, qv.x, L - 1) ? 0.0f : __fdiv_rn(fabsf(g.x), h.x * a0);
            un.y = bcd_blocked(g.y, a1, qv.y, L - 1) ? 0.0f : __fdiv_rn(fabsf(g.y), h.y * a1);
            un.z = bcd_blocked(g.z, a2, qv.z, L - 1) ? 0.0f : __fdiv_rn(fabsf(g.z), h.z * a2);
            un.w = bcd_blocked(g.w, a3, qv.w, L - 1) ? 0.0f : __fdiv_rn(fabsf(g.w), h.w * a3);
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

// ------------------------------------------------------------------------------------------------
// Several columns per workgroup.  Near a coordinate-wise optimum almost every iteration is idle for a
// column; what it costs is reading the iteration's row of the pair table, the test of every pair and a
// barrier.  Here a workgroup of 1024 threads owns CW columns and pays that once for all of them.
//   The pair test.  With u = |2 g| / (H_ii a) per coordinate and rho = |H_ik| / sqrt(H_ii H_kk), a move
//   (di, dk) of the pair changes the loss by at least x^2 (1 - u_i) + y^2 (1 - u_k) - 2 rho x y with
//   x = |di| sqrt(H_ii), y = |dk| sqrt(H_kk), which is >= tau (x^2 + y^2) for all x, y when
//   (1 - u_i - tau)(1 - u_k - tau) >= rho^2 and both factors are >= 0; tau = 2^-14 keeps fp32 rounding of the
//   scores (below 1e-6 of the same magnitude) from turning such a pair into a move.  Both u <= 1 - rho - tau,
//   the one-column kernel's test, implies this one, so fewer pairs are scored here.
//   state in LDS: 2g [coordinate][column] fp32; v = 1 - u - tau in units of 2^-16 rounded DOWN,
//   V [coordinate][column] u16, and its minimum over the columns, Vmin [coordinate]; H_ii; the codes, 4 bits a
//   column in one word a coordinate; a ring of pair-table rows (i | k << 16, 2 H_ik, and rho^2 rounded
//   UP to 16 bits) that direct global->LDS loads fill several iterations ahead.
//   per pair: (vmin_i vmin_k) >> 16 >= R proves the bound for every column (all roundings are on the safe
//   side, by more than fp32 rounding moves u or rho): four small LDS reads, a 24-bit multiply and a compare.
//   Otherwise the two V rows say which columns go to the queue.
//   queue (column, pair): up to BCDM_SPREAD entries 16 lanes share an entry's level pairs, up to the
//   queue's size a thread takes an entry; beyond (far from an optimum) every thread scores its own pairs
//   for every column.  Candidates go straight to the column's 64-bit key (score image, then block and
//   levels) with an LDS minimum, so the result does not depend on the order.
//   commit: the columns that found a move update 2g with two H rows, then V and Vmin.
constexpr int BCDM_NT = 1024;
constexpr int BCDM_QMAX = 512;      // queued entries (column | pair << 4), 4 bytes each
constexpr int BCDM_SPREAD = 128;    // up to this many entries, 16 lanes share an entry's level pairs
constexpr int BCDM_MAXI = 3;        // direct loads of 1 KiB a wavefront issues per pair-table row, at most

// coordinates per thread the kernel is built for; more than the LDS can hold for that many columns (checked again by the host)
constexpr int bcdm_xpt(int cw) { return (cw == 8 ? 3 : cw == 4 ? 4 : 5) * (1024 / BCDM_NT); }

__device__ __forceinline__ void bcdm_wait_vmem(int n) {       // at most n of this wavefront's vector-memory operations pending
    switch (n) {
        case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
        case 1: asm volatile("s_waitcnt vmcnt(1)" ::: "memory"); break;
        case 2: asm volatile("s_waitcnt vmcnt(2)" ::: "memory"); break;
        case 3: asm volatile("s_waitcnt vmcnt(3)" ::: "memory"); break;
        case 4: asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); break;
        case 5: asm volatile("s_waitcnt vmcnt(5)" ::: "memory"); break;
        case 6: asm volatile("s_waitcnt vmcnt(6)" ::: "memory"); break;
        case 7: asm volatile("s_waitcnt vmcnt(7)" ::: "memory"); break;
        case 8: asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); break;
        default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;      // waiting for more than needed is always safe
    }
}

// v = 1 - u - tau in units of 2^-16 (tau is 4 of them), rounded DOWN by more than one unit; 0 when u is not a number
// below 1 - 10 units
__device__ __forceinline__ uint32_t bcdm_v16(float g2, float h, float a, int q, int top) {
    const float u = bcd_blocked(g2, a, q, top) ? 0.0f : __fdiv_rn(fabsf(g2), h * a);
    return (u >= 0.0f && u < 0.99985f) ? 65530u - (uint32_t)(u * 65536.0f) : 0u;
}

// (v_i v_k) >> 16 for two 16-bit margins.  __umul24 returns a signed int: without the cast the shift would smear the sign
// of a product of 2^31 or more over the result, and the pair would pass the test whatever its rho.
__device__ __forceinline__ uint32_t bcdm_margin(uint32_t vi, uint32_t vk) { return (uint32_t)__umul24(vi, vk) >> 16; }

// pair-table rows for the kernel above: ik [T][n_pairs] u32, R [T][n_pairs] u16 = rho^2 in units of 2^-16 rounded UP by more than
// one unit (65535 = never skip)
__global__ __launch_bounds__(256) void bcdm_pair_gather_kernel(const float* __restrict__ H, const int32_t* __restrict__ parts,
                                                               const int32_t* __restrict__ bad, int64_t d_in, int64_t n_items,
                                                               uint32_t* __restrict__ pair_ik, uint16_t* __restrict__ pair_thr,
                                                               float* __restrict__ pair_h2) {
    const int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x;        // x = t * (d_in/2) + p
    if (x >= n_items || *bad != 0) return;                            // indices are only followed once the check accepted them
    const int32_t i = parts[2 * x], k = parts[2 * x + 1];
    const float h2 = 2.0f * H[(int64_t)i * d_in + k];
    const float hii = H[(int64_t)i * d_in + i], hkk = H[(int64_t)k * d_in + k];
    uint32_t r16 = 65535u;
    if (hii > 0.0f && hkk > 0.0f) {
        const float rho = (0.5f * fabsf(h2) * __frsqrt_rn(hii)) * __frsqrt_rn(hkk);
        const float r2 = rho * rho;
        if (r2 < 0.99f) r16 = (uint32_t)(r2 * 65536.0f) + 2u;
    }
    pair_ik[x] = (uint32_t)i | ((uint32_t)k << 16);
    pair_thr[x] = (uint16_t)r16;
    pair_h2[x] = h2;
}

template <int BITS, int CW>
__global__ __launch_bounds__(BCDM_NT) void bcd2_multi_kernel(const float* __restrict__ H, const float* __restrict__ hdiag,
                                                             const float* __restrict__ G0, const float* __restrict__ scale,
                                                             uint8_t* __restrict__ Q, const uint32_t* __restrict__ pair_ik,
                                                             const uint16_t* __restrict__ pair_thr, const float* __restrict__ pair_h2,
                                                             const int32_t* __restrict__ bad_parts,
                                                             int d_out, int d_in, int group, int T, int nst, int score_all,
                                                             int32_t* __restrict__ moves_out, float* __restrict__ G_out,
                                                             int32_t* __restrict__ trace, int trace_cap) {
    constexpr int L = 1 << BITS, NC = L * L;
    constexpr int XPT = bcdm_xpt(CW);                                       // coordinates a thread owns at most
    constexpr int LPE = 16, CPL = NC / LPE;                                 // lanes per entry and level pairs per lane when an entry is shared
    static_assert(NC % LPE == 0, "at least 2 bits");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n_grp = d_in / group, n_pairs = d_in / 2;
    // group of a coordinate without a division: exact for coordinates below 2^16 and groups below 2^13
    const uint32_t grp_mul = (uint32_t)((0x100000000ull + (uint32_t)group - 1u) / (uint32_t)group);
    auto grp = [&](int i) { return group == 1 ? i : (int)__umulhi((uint32_t)i, grp_mul); };
    const int j0 = blockIdx.x * CW;
    const int ncol = (d_out - j0 < CW) ? d_out - j0 : CW;
    const int stage_bytes = 10 * n_pairs;                                   // ik (4 B a pair), 2 H_ik (4 B), thr16 (2 B)
    float* g2 = reinterpret_cast<float*>(smem);                             // [d_in][CW]
    uint16_t* V = reinterpret_cast<uint16_t*>(g2 + (size_t)d_in * CW);      // [d_in][CW]
    float* hd = reinterpret_cast<float*>(V + (size_t)d_in * CW);            // [d_in]
    using qpack_t = typename std::conditional<(CW <= 2), uint8_t, uint32_t>::type;
    qpack_t* qpack = reinterpret_cast<qpack_t*>(hd + d_in);                 // [d_in] 4 bits a column
    char* ring = reinterpret_cast<char*>(qpack + d_in);                     // [nst][stage_bytes]
    int* queue = reinterpret_cast<int*>(ring + (size_t)nst * stage_bytes);  // [BCDM_QMAX] column | pair << 4
    unsigned long long* colkey = reinterpret_cast<unsigned long long*>(queue + BCDM_QMAX);   // [2][CW]
    float* a = reinterpret_cast<float*>(colkey + 2 * CW);                   // [CW][n_grp]
    int* cnt = reinterpret_cast<int*>(a + CW * n_grp);                      // [4] ring of queue lengths
    int* found = cnt + 4;                                                   // [2] set when a column offered a move; [2] spare
    int* moves = cnt + 8;                                                   // [8] committed moves per column, written by thread 0
    uint16_t* Vmin = reinterpret_cast<uint16_t*>(cnt + 16);                 // [d_in]

    if (*bad_parts != 0) {                                                  // invalid partitions: leave the columns untouched
        if (tid < ncol && moves_out != nullptr) moves_out[j0 + tid] = -1;
        return;
    }
    for (int x = tid; x < CW * n_grp; x += BCDM_NT) {
        const int c = x / n_grp;
        a[x] = (c < ncol) ? scale[(int64_t)(j0 + c) * n_grp + x % n_grp] : 1.0f;
    }
    if (tid < 16) cnt[tid] = 0;
    if (tid < 2 * CW) colkey[tid] = ~0ull;
    for (int i = tid; i < d_in; i += BCDM_NT) hd[i] = hdiag[i];
    __syncthreads();
    for (int i = tid; i < d_in; i += BCDM_NT) {                             // a thread owns coordinate i in all columns
        uint32_t qp = 0, vm = 65535u;
        const float h = hd[i];
        float gl[CW];
        uint32_t ql[CW];
#pragma unroll
        for (int c = 0; c < CW; ++c) {                                      // columns past the end load column 0: every load is in flight at once
            const int64_t col = j0 + (c < ncol ? c : 0);
            gl[c] = G0[col * d_in + i];
            ql[c] = Q[col * d_in + i];
        }
#pragma unroll
        for (int c = 0; c < CW; ++c) {
            const float g = (c < ncol) ? 2.0f * gl[c] : 0.0f;
            const uint32_t qv = (c < ncol) ? ql[c] : 0u;
            const uint32_t u = (c < ncol) ? bcdm_v16(g, h, a[c * n_grp + grp(i)], (int)qv, L - 1) : 65535u;
            g2[i * CW + c] = g;
            V[i * CW + c] = (uint16_t)u;
            qp |= qv << (4 * c);
            vm = vm < u ? vm : u;
        }
        qpack[i] = (qpack_t)qp;
        Vmin[i] = (uint16_t)vm;
    }

    // ---- ring of pair-table rows: 16-byte chunk x of a stage comes from ik, 2 H_ik or thr16
    const int ch_ik = n_pairs / 4, ch_h2 = n_pairs / 4, chunks = ch_ik + ch_h2 + n_pairs / 8;
    const int n_instr = (chunks + 63) / 64;
    const int my_instr = (n_instr > wave) ? (n_instr - wave + BCDM_NT / 64 - 1) / (BCDM_NT / 64) : 0;   // direct loads this wavefront issues per stage
    const uint32_t ring_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)ring;
    // a wavefront issues at most BCDM_MAXI loads a stage (the host checks it): per lane the source of row 0 and the bytes
    // from one row to the next are fixed, per wavefront the offset in the stage
    const char* src0[BCDM_MAXI];
    uint32_t row_step[BCDM_MAXI], lds_off[BCDM_MAXI];
    bool on[BCDM_MAXI];
#pragma unroll
    for (int s2 = 0; s2 < BCDM_MAXI; ++s2) {
        const int ii = wave + (BCDM_NT / 64) * s2, x = ii * 64 + lane;
        on[s2] = ii < n_instr && x < chunks;
        const int arr = (x < ch_ik) ? 0 : (x < ch_ik + ch_h2) ? 1 : 2;
        const char* base = arr == 0 ? reinterpret_cast<const char*>(pair_ik) : arr == 1 ? reinterpret_cast<const char*>(pair_h2)
                                                                                        : reinterpret_cast<const char*>(pair_thr);
        src0[s2] = base + 16 * (int64_t)(arr == 0 ? x : arr == 1 ? x - ch_ik : x - ch_ik - ch_h2);
        row_step[s2] = (uint32_t)n_pairs * (arr == 2 ? 2u : 4u);
        lds_off[s2] = (uint32_t)(ii * 1024);
    }
    auto issue = [&](int t, int stage_idx) {
        const uint32_t stage_lds = ring_lds + (uint32_t)(stage_idx * stage_bytes);
#pragma unroll
        for (int s2 = 0; s2 < BCDM_MAXI; ++s2) {
            const char* src = src0[s2] + (uint64_t)row_step[s2] * (uint32_t)t;
            const uint32_t m0v = __builtin_amdgcn_readfirstlane(stage_lds + lds_off[s2]);
            if (on[s2])
                asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(m0v), "v"(src) : "m0", "memory");
        }
    };
    const int pro = (T < nst - 1) ? T : nst - 1;
    for (int t = 0; t < pro; ++t) issue(t, t);
    bcdm_wait_vmem((pro - 1) * my_instr);                        // the first row has landed
    __syncthreads();

    const uint32_t valid_mask = (1u << ncol) - 1u;

    int st_cur = 0, st_fill = nst - 1;                            // stage of iteration t; stage the next load goes to (that of t - 1)
    const int steady_wait = (nst - 3) * my_instr;
    for (int t = 0; t < T; ++t, st_cur = (st_cur + 1 == nst) ? 0 : st_cur + 1, st_fill = (st_fill + 1 == nst) ? 0 : st_fill + 1) {
        const char* stage = ring + (size_t)st_cur * stage_bytes;
        const uint32_t* s_ik = reinterpret_cast<const uint32_t*>(stage);
        const float* s_h2 = reinterpret_cast<const float*>(stage + 4 * (size_t)n_pairs);
        const uint16_t* s_thr = reinterpret_cast<const uint16_t*>(stage + 8 * (size_t)n_pairs);
        int* my_cnt = cnt + (t & 3);
        unsigned long long* key_t = colkey + (t & 1) * CW;
        // level pair cidx = r_i * L + r_k of pair p for column c
        auto score_one = [&](int c, int p, int i, int k, float hh, float ai, float ak, float gi, float gk, float hii, float hkk,
                             int qi, int qk, int cidx, float& best_s, uint32_t& best_pay) {
            const int ri = cidx >> BITS, rk = cidx & (L - 1);
            const float di = ai * (float)(ri - qi), dk = ak * (float)(rk - qk);
            const float si = di * fmaf(di, hii, gi), sk = dk * fmaf(dk, hkk, gk);
            const float sc = fmaf(di * dk, hh, si + sk);
            if (sc < best_s) { best_s = sc; best_pay = ((uint32_t)p << 8) | (uint32_t)(ri << 4) | (uint32_t)rk; }
        };
        // level pairs sub, sub + step, ... of pair p for column c in increasing order, folded into the running best
        auto score_pair = [&](int c, int p, int sub, int step, float& best_s, uint32_t& best_pay) {
            const uint32_t ik = s_ik[p];
            const int i = (int)(ik & 0xffffu), k = (int)(ik >> 16);
            const float hh = s_h2[p];
            const float ai = a[c * n_grp + grp(i)], ak = a[c * n_grp + grp(k)];
            const float gi = g2[i * CW + c], gk = g2[k * CW + c], hii = hd[i], hkk = hd[k];
            const int qi = (int)((qpack[i] >> (4 * c)) & 15u), qk = (int)((qpack[k] >> (4 * c)) & 15u);
            if (step == 1) {
#pragma unroll
                for (int cidx = 0; cidx < NC; ++cidx) score_one(c, p, i, k, hh, ai, ak, gi, gk, hii, hkk, qi, qk, cidx, best_s, best_pay);
            } else {
#pragma unroll
                for (int m = 0; m < CPL; ++m) score_one(c, p, i, k, hh, ai, ak, gi, gk, hii, hkk, qi, qk, sub + m * LPE, best_s, best_pay);
            }
        };
        auto offer = [&](int c, float best_s, uint32_t best_pay) {
            if (best_s < 0.0f) {
                const unsigned long long key = ((unsigned long long)order_bits(best_s) << 32) | best_pay;
                if (key < key_t[c]) {
                    found[t & 1] = 1;
                    atomicMin(&key_t[c], key);
                }
            }
        };

        // ---- which (column, pair) need scoring
        for (int p = tid; p < n_pairs; p += BCDM_NT) {
            const uint32_t ik = s_ik[p];
            const uint32_t thr = s_thr[p];
            const int i = (int)(ik & 0xffffu), k = (int)(ik >> 16);
            const uint32_t vi = Vmin[i], vk = Vmin[k];
            if (bcdm_margin(vi, vk) < thr || score_all) {
                uint32_t mask = 0;
#pragma unroll
                for (int c = 0; c < CW; ++c) mask |= (bcdm_margin(V[i * CW + c], V[k * CW + c]) < thr ? 1u : 0u) << c;
                if (score_all) mask = ~0u;
                mask &= valid_mask;
                if (mask) {
                    int pos = atomicAdd(my_cnt, __builtin_popcount(mask));
                    while (mask) {
                        const int c = __builtin_ctz(mask);
                        mask &= mask - 1;
                        if (pos < BCDM_QMAX) queue[pos] = c | (p << 4);
                        ++pos;
                    }
                }
            }
        }
        // the next iteration's row has landed when only the loads issued after it are pending (loads return in order);
        // near the end fewer were issued and everything is waited for
        if (t + nst - 1 <= T) bcdm_wait_vmem(steady_wait);
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();                                         // the queue is complete, the next row visible, iteration t-1 over for everybody
        if (t + nst - 1 < T) issue(t + nst - 1, st_fill);        // into the stage iteration t-1 read
        if (tid == 0) { cnt[(t + 2) & 3] = 0; found[(t + 1) & 1] = 0; }
        if (tid < CW) colkey[((t + 1) & 1) * CW + tid] = ~0ull;
        const int n_q = *my_cnt;
        if (n_q == 0) continue;                                  // an idle iteration costs one barrier

        if (n_q <= BCDM_SPREAD) {
            // ---- few: 16 lanes share an entry
            for (int x = tid / LPE; x < n_q; x += BCDM_NT / LPE) {
                const int e = queue[x];
                float best_s = 0.0f;
                uint32_t best_pay = 0xffffffffu;
                score_pair(e & 15, e >> 4, tid % LPE, LPE, best_s, best_pay);
                offer(e & 15, best_s, best_pay);
            }
        } else if (n_q <= BCDM_QMAX) {
            // ---- more: an entry per thread
            for (int x = tid; x < n_q; x += BCDM_NT) {
                const int e = queue[x];
                float best_s = 0.0f;
                uint32_t best_pay = 0xffffffffu;
                score_pair(e & 15, e >> 4, 0, 1, best_s, best_pay);
                offer(e & 15, best_s, best_pay);
            }
        } else {
            // ---- the queue overflowed: every thread scores its own pairs for every column
            for (int c = 0; c < ncol; ++c) {
                float best_s = 0.0f;
                uint32_t best_pay = 0xffffffffu;
                for (int p = tid; p < n_pairs; p += BCDM_NT) score_pair(c, p, 0, 1, best_s, best_pay);
                const uint64_t key = wave_min_key(order_bits(best_s), best_pay);
                if (lane == 0 && (uint32_t)(key >> 32) < kOrderedZero) {
                    found[t & 1] = 1;
                    atomicMin(&key_t[c], (unsigned long long)key);
                }
            }
        }
        __syncthreads();                                         // the columns' keys are final
        if (found[t & 1] == 0) continue;                         // scored, no move: two barriers
        // ---- commit: every thread derives the moves, then updates its own coordinates of 2g, V and Vmin
        bool any = false;
        for (int c = 0; c < ncol; ++c) {                       // a loop, not unrolled: moves are rare and the code is long
            const unsigned long long key = key_t[c];
            if ((uint32_t)(key >> 32) < kOrderedZero) {
                any = true;
                const uint32_t pay = (uint32_t)key;
                const int p = (int)(pay >> 8), ri = (int)((pay >> 4) & 15u), rk = (int)(pay & 15u);
                const uint32_t ik = s_ik[p];
                const int i = (int)(ik & 0xffffu), k = (int)(ik >> 16);
                const float di2 = 2.0f * (a[c * n_grp + grp(i)] * (float)(ri - (int)((qpack[i] >> (4 * c)) & 15u)));
                const float dk2 = 2.0f * (a[c * n_grp + grp(k)] * (float)(rk - (int)((qpack[k] >> (4 * c)) & 15u)));
                const float* hi = H + (int64_t)i * d_in;
                const float* hk = H + (int64_t)k * d_in;
                float hiv[XPT], hkv[XPT];                       // both rows' loads in flight together (d_in <= XPT * BCDM_NT here)
#pragma unroll
                for (int xx = 0; xx < XPT; ++xx) {
                    const int x = tid + xx * BCDM_NT, xc = x < d_in ? x : 0;
                    hiv[xx] = hi[xc];
                    hkv[xx] = hk[xc];
                }
#pragma unroll
                for (int xx = 0; xx < XPT; ++xx) {
                    const int x = tid + xx * BCDM_NT;
                    if (x < d_in) {
                        const float g = fmaf(dk2, hkv[xx], fmaf(di2, hiv[xx], g2[x * CW + c]));
                        g2[x * CW + c] = g;
                        const int qx = x == i ? ri : x == k ? rk : (int)((qpack[x] >> (4 * c)) & 15u);   // the codes after this move
                        V[x * CW + c] = (uint16_t)bcdm_v16(g, hd[x], a[c * n_grp + grp(x)], qx, L - 1);
                    }
                }
            }
        }
        // every load of the commit has landed (a load whose result a thread did not use would otherwise count as
        // pending at the loop head and make the compiler wait for vector memory, and with it for the ring's loads)
        __builtin_amdgcn_s_waitcnt(0x0F70);                      // vmcnt(0) only
        if (any)
            for (int x = tid; x < d_in; x += BCDM_NT) {
                uint32_t vm = 65535u;
#pragma unroll
                for (int c = 0; c < CW; ++c) { const uint32_t v = V[x * CW + c]; vm = vm < v ? vm : v; }
                Vmin[x] = (uint16_t)vm;
            }
        __syncthreads();                                         // 2g, V, Vmin are updated and everybody has read the old codes
        if (any && tid == 0) {
            for (int c = 0; c < ncol; ++c) {
                const unsigned long long key = key_t[c];
                if ((uint32_t)(key >> 32) < kOrderedZero) {
                    {
                        const uint32_t pay = (uint32_t)key;
                        const uint32_t ik = s_ik[pay >> 8];
                        const int i = (int)(ik & 0xffffu), k = (int)(ik >> 16);
                        qpack[i] = (qpack_t)((qpack[i] & ~(15u << (4 * c))) | (((pay >> 4) & 15u) << (4 * c)));
                        qpack[k] = (qpack_t)((qpack[k] & ~(15u << (4 * c))) | ((pay & 15u) << (4 * c)));
                        if (trace != nullptr && moves[c] < trace_cap) {
                            int32_t* tr = trace + ((int64_t)(j0 + c) * trace_cap + moves[c]) * 4;
                            tr[0] = t; tr[1] = (int32_t)(pay >> 8);
                            tr[2] = (int32_t)(((pay >> 4) & 15u) | ((pay & 15u) << 4));
                            tr[3] = (int32_t)~(uint32_t)(key >> 32);       // the ordered image of a negative score is ~bits
                        }
                    }
                    ++moves[c];
                }
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    for (int c = 0; c < ncol; ++c)
        for (int i = tid; i < d_in; i += BCDM_NT) {
            Q[(int64_t)(j0 + c) * d_in + i] = (uint8_t)((qpack[i] >> (4 * c)) & 15u);
            if (G_out != nullptr) G_out[(int64_t)(j0 + c) * d_in + i] = 0.5f * g2[i * CW + c];
        }
    if (tid == 0 && moves_out != nullptr) {
#pragma unroll
        for (int c = 0; c < CW; ++c)
            if (c < ncol) moves_out[j0 + c] = moves[c];
    }
}

size_t bcdm_lds_bytes(int64_t d_in, int64_t group, int cw, int nst) {
    const int64_t n_grp = d_in / group, n_pairs = d_in / 2;
    return cdq_align_up((size_t)d_in * cw * 6 + (size_t)d_in * (cw <= 2 ? 7 : 10) + (size_t)nst * 10 * n_pairs + 4 * BCDM_QMAX +
                        sizeof(unsigned long long) * 2 * cw + sizeof(float) * cw * n_grp + sizeof(int) * 16, 16);
}

// ------------------------------------------------------------------------------------------------
// Wide layers (d_in above what the kernels above hold, up to 65534; any alignment).  A 1024-thread workgroup owns
// up to 16 columns (rows of CW in {16, 8, 4, 2, 1} margins).  What bounds an idle iteration here is the two scattered LDS reads per pair of the test,
// so LDS holds only what that test reads for all the columns at once -- the minimum over the columns of v = 1 - u - tau,
// 16 bits a coordinate -- and one pass over the pairs serves CW columns.  Everything else stays in global memory: the
// per-column v (rows of CW values, read for the few pairs that fail the test on the minimum), 2g (the workspace's
// gradient rows, doubled in place), H_ii, the step sizes and the codes; from a coordinate-wise optimum few pairs are
// scored and fewer commit, so those reads are rare.  The pair table is the several-column kernel's (i | k << 16, rho^2
// in 16 bits rounded up, 2 H_ik) and so is the test, (vmin_i vmin_k) >> 16 >= R; a thread reads 6 bytes of table per
// pair, one batch of entries ahead of the one it tests.
// Per iteration: test -> queue of (column, pair) -> barrier -> (if any) score the queue, 16 lanes an entry, candidates
// to the column's 64-bit key by an LDS minimum -> barrier -> (if a column found a move) commit.
constexpr int BCDW_NT = 1024;
constexpr int BCDW_UNR = 8;          // table entries whose loads are in flight together, per thread
constexpr int BCDW_QMAX = 512;
constexpr int BCDW_SPREAD = 128;
constexpr int BCDW_CUNR = 6;         // coordinates per thread whose loads are in flight together at a commit

// the CW 16-bit margins of one coordinate, one load
template <int CW>
__device__ __forceinline__ void bcdw_load_row(const uint16_t* p, uint32_t (&v)[CW]) {
    if constexpr (CW == 16) {
        const uint4 w0 = *reinterpret_cast<const uint4*>(p), w1 = *reinterpret_cast<const uint4*>(p + 8);
        v[0] = w0.x & 0xffffu; v[1] = w0.x >> 16; v[2] = w0.y & 0xffffu; v[3] = w0.y >> 16;
        v[4] = w0.z & 0xffffu; v[5] = w0.z >> 16; v[6] = w0.w & 0xffffu; v[7] = w0.w >> 16;
        v[8] = w1.x & 0xffffu; v[9] = w1.x >> 16; v[10] = w1.y & 0xffffu; v[11] = w1.y >> 16;
        v[12] = w1.z & 0xffffu; v[13] = w1.z >> 16; v[14] = w1.w & 0xffffu; v[15] = w1.w >> 16;
    } else if constexpr (CW == 8) {
        const uint4 w = *reinterpret_cast<const uint4*>(p);
        v[0] = w.x & 0xffffu; v[1] = w.x >> 16; v[2] = w.y & 0xffffu; v[3] = w.y >> 16;
        v[4] = w.z & 0xffffu; v[5] = w.z >> 16; v[6] = w.w & 0xffffu; v[7] = w.w >> 16;
    } else if constexpr (CW == 4) {
        const uint2 w = *reinterpret_cast<const uint2*>(p);
        v[0] = w.x & 0xffffu; v[1] = w.x >> 16; v[2] = w.y & 0xffffu; v[3] = w.y >> 16;
    } else if constexpr (CW == 2) {
        const uint32_t w = *reinterpret_cast<const uint32_t*>(p);
        v[0] = w & 0xffffu; v[1] = w >> 16;
    } else {
        v[0] = *p;
    }
}

template <int BITS, int CW>
__global__ __launch_bounds__(BCDW_NT) void bcd2_wide_kernel(const float* __restrict__ H, const float* __restrict__ hdiag, float* G2,
                                                            uint16_t* Vg_all, const float* __restrict__ scale, uint8_t* Q,
                                                            const uint32_t* __restrict__ pair_ik, const uint16_t* __restrict__ pair_thr,
                                                            const float* __restrict__ pair_h2, const int32_t* __restrict__ bad_parts,
                                                            int d_out, int d_in, int group, int T, int cpw, int score_all,
                                                            int32_t* __restrict__ moves_out, float* __restrict__ G_out,
                                                            int32_t* __restrict__ trace, int trace_cap) {
    constexpr int L = 1 << BITS, NC = L * L;
    constexpr int LPE = 16, CPL = NC / LPE;
    constexpr int CUNR = CW > 8 ? 3 : BCDW_CUNR;                  // fewer coordinates in flight at a commit where a row of margins is long
    extern __shared__ __attribute__((aligned(16))) char smem[];
    __shared__ unsigned long long colkey[3][CW];                  // per iteration mod 3: the columns' best (score image, pair, levels)
    __shared__ int cnt[4];                                        // ring of queue lengths
    __shared__ int found[3];                                      // per iteration mod 3: some column offered a move
    __shared__ int moves[CW];
    __shared__ int queue[BCDW_QMAX];                              // column | pair << 4
    __shared__ uint32_t queue_ik[BCDW_QMAX];                      // the pair's i | k << 16
    uint16_t* Vmin = reinterpret_cast<uint16_t*>(smem);           // [d_in] min over the columns of v
    uint16_t* V = Vg_all + (size_t)blockIdx.x * d_in * CW;        // [d_in][CW] in global memory, this workgroup's alone
    const int tid = threadIdx.x, lane = tid & 63;
    const int n_grp = d_in / group, n_pairs = d_in / 2;
    const uint32_t grp_mul = (uint32_t)((0x100000000ull + (uint32_t)group - 1u) / (uint32_t)group);   // exact below 2^16 (group > 1)
    auto grp = [&](int i) { return n_grp == 1 ? 0 : (group == 1 ? i : (int)__umulhi((uint32_t)i, grp_mul)); };
    const int j0 = blockIdx.x * cpw;                              // cpw <= CW columns per workgroup; rows of margins are CW long
    const int ncol = (d_out - j0 < cpw) ? d_out - j0 : cpw;
    if (*bad_parts != 0) {                                        // invalid partitions: leave the columns untouched
        if (tid < ncol && moves_out != nullptr) moves_out[j0 + tid] = -1;
        return;
    }
    if (tid < 3 * CW) (&colkey[0][0])[tid] = ~0ull;
    if (tid < 4) cnt[tid] = 0;
    if (tid < 3) found[tid] = 0;
    if (tid < CW) moves[tid] = 0;
    for (int i = tid; i < d_in; i += BCDW_NT) {                   // a thread owns coordinate i in all columns
        const float h = hdiag[i];
        uint32_t vm = 65535u;
#pragma unroll
        for (int c = 0; c < CW; ++c) {
            uint32_t v = 65535u;                                  // columns past the end never fail the test
            if (c < ncol) {
                const int64_t at = (int64_t)(j0 + c) * d_in + i;
                const float g = 2.0f * G2[at];
                G2[at] = g;                                       // from here on the row holds 2g
                v = bcdm_v16(g, h, scale[(int64_t)(j0 + c) * n_grp + grp(i)], (int)Q[at], L - 1);
            }
            if (CW > 1) V[(size_t)i * CW + c] = (uint16_t)v;
            vm = vm < v ? vm : v;
        }
        Vmin[i] = (uint16_t)vm;
    }
    __syncthreads();

    const uint32_t valid_mask = (1u << ncol) - 1u;
    // table entries travel through registers one batch ahead: the next batch of this iteration, or the first of the next one,
    // is requested before the current batch is tested, so an idle iteration does not wait for memory after its barrier
    uint32_t nik[BCDW_UNR], nthr[BCDW_UNR];
    auto fetch = [&](int tt, int p0) {
        const uint32_t* f_ik = pair_ik + (int64_t)tt * n_pairs;
        const uint16_t* f_thr = pair_thr + (int64_t)tt * n_pairs;
#pragma unroll
        for (int u = 0; u < BCDW_UNR; ++u) {                      // entries past the end reload the batch's first one
            const int p = p0 + u * BCDW_NT, pc = p < n_pairs ? p : p0;
            nik[u] = f_ik[pc];
            nthr[u] = f_thr[pc];
        }
    };
    if (tid < n_pairs) fetch(0, tid);
    for (int t = 0; t < T; ++t) {
        const int64_t row = (int64_t)t * n_pairs;
        const uint32_t* r_ik = pair_ik + row;
        const float* r_h2 = pair_h2 + row;
        int* my_cnt = cnt + (t & 3);
        unsigned long long* key_t = colkey[t % 3];
        int* found_t = found + t % 3;
        // level pairs sub, sub + step, ... of pair p for column c in increasing order (r_i major), folded into the running best
        auto score_pair = [&](int c, int p, uint32_t ik, int sub, int step, float& best_s, uint32_t& best_pay) {
            const int i = (int)(ik & 0xffffu), k = (int)(ik >> 16);
            const int64_t col = j0 + c;
            const float hh = r_h2[p];
            const float ai = scale[col * n_grp + grp(i)], ak = scale[col * n_grp + grp(k)];
            const float gi = G2[col * d_in + i], gk = G2[col * d_in + k], hii = hdiag[i], hkk = hdiag[k];
            const int qi = Q[col * d_in + i], qk = Q[col * d_in + k];
            auto one = [&](int cidx) {
                const int ri = cidx >> BITS, rk = cidx & (L - 1);
                const float di = ai * (float)(ri - qi), dk = ak * (float)(rk - qk);
                const float si = di * fmaf(di, hii, gi), sk = dk * fmaf(dk, hkk, gk);
                const float sc = fmaf(di * dk, hh, si + sk);
                if (sc < best_s) { best_s = sc; best_pay = ((uint32_t)p << 8) | (uint32_t)(ri << 4) | (uint32_t)rk; }
            };
            if (step == 1) {
#pragma unroll
                for (int m = 0; m < NC; ++m) one(m);
            } else {
#pragma unroll
                for (int m = 0; m < CPL; ++m) one(sub + m * LPE);
            }
        };
        auto offer = [&](int c, float best_s, uint32_t best_pay) {
            if (best_s < 0.0f) {
                const unsigned long long key = ((unsigned long long)order_bits(best_s) << 32) | best_pay;
                *found_t = 1;
                atomicMin(&key_t[c], key);
            }
        };

        // ---- which (column, pair) need scoring
        for (int p0 = tid; p0 < n_pairs; p0 += BCDW_NT * BCDW_UNR) {
            uint32_t ik[BCDW_UNR], thr[BCDW_UNR];
#pragma unroll
            for (int u = 0; u < BCDW_UNR; ++u) { ik[u] = nik[u]; thr[u] = nthr[u]; }
            if (p0 + BCDW_NT * BCDW_UNR < n_pairs) fetch(t, p0 + BCDW_NT * BCDW_UNR);
            else if (t + 1 < T) fetch(t + 1, tid);
#pragma unroll
            for (int u = 0; u < BCDW_UNR; ++u) {
                const int p = p0 + u * BCDW_NT;
                const int i = (int)(ik[u] & 0xffffu), k = (int)(ik[u] >> 16);
                const uint32_t vi = Vmin[i], vk = Vmin[k];
                if (p < n_pairs && (bcdm_margin(vi, vk) < thr[u] || score_all)) {
                    uint32_t mask = 1u;
                    if (CW > 1) {                                 // which columns: their own margins, two rows from global memory
                        uint32_t ri[CW], rk[CW];
                        bcdw_load_row<CW>(V + (size_t)i * CW, ri);
                        bcdw_load_row<CW>(V + (size_t)k * CW, rk);
                        mask = 0u;
#pragma unroll
                        for (int c = 0; c < CW; ++c) mask |= (bcdm_margin(ri[c], rk[c]) < thr[u] ? 1u : 0u) << c;
                    }
                    if (score_all) mask = ~0u;
                    mask &= valid_mask;
                    if (mask) {
                        int pos = atomicAdd(my_cnt, __builtin_popcount(mask));
                        while (mask) {
                            const int c = __builtin_ctz(mask);
                            mask &= mask - 1;
                            if (pos < BCDW_QMAX) { queue[pos] = c | (p << 4); queue_ik[pos] = ik[u]; }
                            ++pos;
                        }
                    }
                }
            }
        }
        __syncthreads();                                         // the queue is complete; iteration t-1 is over for everybody
        if (tid == 0) { cnt[(t + 2) & 3] = 0; found[(t + 2) % 3] = 0; }
        if (tid < CW) colkey[(t + 2) % 3][tid] = ~0ull;
        const int n_q = *my_cnt;
        if (n_q == 0) continue;                                  // an idle iteration costs one barrier

        if (n_q <= BCDW_SPREAD) {
            for (int x = tid / LPE; x < n_q; x += BCDW_NT / LPE) {                  // few: 16 lanes share an entry
                const int e = queue[x];
                float best_s = 0.0f;
                uint32_t best_pay = 0xffffffffu;
                score_pair(e & 15, e >> 4, queue_ik[x], tid % LPE, LPE, best_s, best_pay);
                offer(e & 15, best_s, best_pay);
            }
        } else if (n_q <= BCDW_QMAX) {
            for (int x = tid; x < n_q; x += BCDW_NT) {                              // more: an entry per thread
                const int e = queue[x];
                float best_s = 0.0f;
                uint32_t best_pay = 0xffffffffu;
                score_pair(e & 15, e >> 4, queue_ik[x], 0, 1, best_s, best_pay);
                offer(e & 15, best_s, best_pay);
            }
        } else {
            for (int c = 0; c < ncol; ++c) {                                        // the queue overflowed: everything, column by column
                float best_s = 0.0f;
                uint32_t best_pay = 0xffffffffu;
                for (int p = tid; p < n_pairs; p += BCDW_NT) score_pair(c, p, r_ik[p], 0, 1, best_s, best_pay);
                const uint64_t key = wave_min_key(order_bits(best_s), best_pay);
                if (lane == 0 && (uint32_t)(key >> 32) < kOrderedZero) {
                    *found_t = 1;
                    atomicMin(&key_t[c], (unsigned long long)key);
                }
            }
        }
        __syncthreads();                                         // the columns' keys are final
        if (*found_t == 0) continue;                             // scored, no move: two barriers
        // ---- commit: every thread derives the moves, then updates its own coordinates of 2g, V and Vmin for the moving
        // columns, one after the other
        for (int c = 0; c < ncol; ++c) {
            const unsigned long long key = key_t[c];
            if ((uint32_t)(key >> 32) >= kOrderedZero) continue;
            const uint32_t pay = (uint32_t)key;
            const int p = (int)(pay >> 8), ri = (int)((pay >> 4) & 15u), rk = (int)(pay & 15u);
            const uint32_t ik = r_ik[p];
            const int i = (int)(ik & 0xffffu), k = (int)(ik >> 16);
            const int64_t col = j0 + c;
            float* g2c = G2 + col * d_in;
            const uint8_t* qc = Q + col * d_in;
            const float* ac = scale + col * n_grp;
            const float di2 = 2.0f * (ac[grp(i)] * (float)(ri - (int)qc[i])), dk2 = 2.0f * (ac[grp(k)] * (float)(rk - (int)qc[k]));
            const float* hi = H + (int64_t)i * d_in;
            const float* hk = H + (int64_t)k * d_in;
            for (int x0 = tid; x0 < d_in; x0 += BCDW_NT * CUNR) {
                float vi[CUNR], vk[CUNR], gv[CUNR], hv[CUNR], av[CUNR];
                int qv[CUNR];
                uint32_t rows[CUNR][CW];
#pragma unroll
                for (int u = 0; u < CUNR; ++u) {             // all loads of a batch of coordinates in flight together
                    const int x = x0 + u * BCDW_NT, xc = x < d_in ? x : x0;
                    vi[u] = hi[xc]; vk[u] = hk[xc]; gv[u] = g2c[xc]; hv[u] = hdiag[xc]; av[u] = ac[grp(xc)]; qv[u] = qc[xc];
                    if (CW > 1) bcdw_load_row<CW>(V + (size_t)xc * CW, rows[u]);
                }
#pragma unroll
                for (int u = 0; u < CUNR; ++u) {
                    const int x = x0 + u * BCDW_NT;
                    if (x < d_in) {
                        const float g = fmaf(dk2, vk[u], fmaf(di2, vi[u], gv[u]));
                        g2c[x] = g;
                        const int qx = x == i ? ri : x == k ? rk : qv[u];                   // the codes after this move
                        const uint32_t v = bcdm_v16(g, hv[u], av[u], qx, L - 1);
                        uint32_t vm = v;
                        if (CW > 1) {                             // the row with this column replaced: the new minimum
                            V[(size_t)x * CW + c] = (uint16_t)v;
#pragma unroll
                            for (int c2 = 0; c2 < CW; ++c2) {
                                const uint32_t o = c2 == c ? v : rows[u][c2];
                                vm = vm < o ? vm : o;
                            }
                        }
                        Vmin[x] = (uint16_t)vm;
                    }
                }
            }
            __syncthreads();                                     // (the same keys for every thread: a uniform barrier) this column's
        }                                                        // margins are written before another column's pass reads the rows,
        if (tid == 0) {                                          // and everybody has read the old codes
            for (int c = 0; c < ncol; ++c) {
                const unsigned long long key = key_t[c];
                if ((uint32_t)(key >> 32) >= kOrderedZero) continue;
                const uint32_t pay = (uint32_t)key;
                const uint32_t ik = r_ik[pay >> 8];
                uint8_t* qc = Q + (int64_t)(j0 + c) * d_in;
                qc[ik & 0xffffu] = (uint8_t)((pay >> 4) & 15u);
                qc[ik >> 16] = (uint8_t)(pay & 15u);
                if (trace != nullptr && moves[c] < trace_cap) {
                    int32_t* tr = trace + ((int64_t)(j0 + c) * trace_cap + moves[c]) * 4;
                    tr[0] = t; tr[1] = (int32_t)(pay >> 8);
                    tr[2] = (int32_t)(((pay >> 4) & 15u) | ((pay & 15u) << 4));
                    tr[3] = (int32_t)~(uint32_t)(key >> 32);               // the ordered image of a negative score is ~bits
                }
                ++moves[c];
            }
        }
        __syncthreads();                                         // 2g, V, Vmin and the codes are updated
    }
    __syncthreads();
    for (int c = 0; c < ncol; ++c) {
        if (G_out != nullptr)
            for (int i = tid; i < d_in; i += BCDW_NT) G_out[(int64_t)(j0 + c) * d_in + i] = 0.5f * G2[(int64_t)(j0 + c) * d_in + i];
        if (tid == 0 && moves_out != nullptr) moves_out[j0 + c] = moves[c];
    }
}

size_t bcdw_lds_bytes(int64_t d_in) { return cdq_align_up((size_t)d_in * 2, 16); }

size_t bcd_lds_bytes(int64_t d_in, int64_t group) {
    const int64_t n_grp = d_in / group;
    return cdq_align_up(sizeof(float) * 3 * d_in + 16 * BCD_FASTQ + sizeof(uint64_t) * 32 + sizeof(float) * 8 + sizeof(int) * 4 +
                        sizeof(float) * n_grp + (size_t)d_in, 16);
}

}  // namespace

// workspace: G0 [d_out][d_in] fp32 | hdiag [d_in] | pair table, 12 bytes per (iteration, pair) | flag |
// the wide-layer kernel's 16-bit margins, a row of up to 16 per coordinate and workgroup: at most [2 d_out + 16][d_in].
// (pair_rec int2 + pair_h2 for the one-column kernel, ik + R16 + 2 spare + pair_h2 for the others)
size_t bcd_workspace_bytes(int64_t d_out, int64_t d_in, int64_t T) {
    return cdq_align_up((size_t)d_out * d_in * sizeof(float), 256) + cdq_align_up((size_t)d_in * sizeof(float), 256) +
           cdq_align_up((size_t)T * (d_in / 2) * 12, 256) + 256 +
           cdq_align_up((size_t)(2 * d_out + 16) * d_in * sizeof(uint16_t), 256);
}

int bcd_launch(const float* H, const float* Wt, const float* scale, const float* zero, uint8_t* Q, int64_t d_out, int64_t d_in,
               int bits, int64_t group, const int32_t* parts, int64_t T, int32_t* moves, float* G_out, int32_t* trace,
               int64_t trace_cap, int flags, void* ws, size_t ws_bytes, hipStream_t st) {
    const bool score_all = (flags & 1) != 0, single = (flags & 2) != 0, wide = (flags & 4) != 0;
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
    // one column per workgroup with its state in LDS; failing that, the wide-layer kernel (any alignment)
    const bool single_ok = nt <= 1024 && lds <= 160 * 1024 && d_in % 4 == 0 && ((uintptr_t)H & 15) == 0;
    // wide-layer kernel: cpw columns per workgroup, chosen so that the workgroups fill the 256 CUs a whole number of times
    // (one workgroup per CU at a time), at most 16; its rows of margins are wcw = 1, 2, 4, 8 or 16 long.  The flag keeps 8.
    int wcw = 0, cpw = 0;
    if (d_in < 65536 && bcdw_lds_bytes(d_in) + 4096 <= 160 * 1024) {
        if (wide) cpw = 8;
        else
            for (int64_t k = 1; cpw == 0; ++k) {
                const int64_t c = (d_out + 256 * k - 1) / (256 * k);
                if (c <= 16) cpw = (int)c;
            }
        wcw = cpw > 8 ? 16 : cpw > 4 ? 8 : cpw > 2 ? 4 : cpw;
    }
    const bool wide_ok = wcw != 0;
    if ((!single_ok && !wide_ok) || T > 0x7fffffffLL || d_out > 0x7fffffffLL) return CDQ_EUNSUPPORTED;
    if (ws == nullptr || ((uintptr_t)ws & 255) || ws_bytes < bcd_workspace_bytes(d_out, d_in, T)) return CDQ_EWORKSPACE;
    const int64_t n_items = T * (d_in / 2);
    char* wp = (char*)ws;
    float* G0 = (float*)wp;           wp += cdq_align_up((size_t)d_out * d_in * sizeof(float), 256);
    float* hdiag = (float*)wp;        wp += cdq_align_up((size_t)d_in * sizeof(float), 256);
    char* table = wp;                 wp += cdq_align_up((size_t)n_items * 12, 256);
    int2* pair_rec = (int2*)table;                                       // [n_items] 8 bytes each, then
    float* pair_h2 = (float*)(table + 8 * (size_t)n_items);              // [n_items]
    int32_t* bad = (int32_t*)wp;       wp += 256;
    uint16_t* Vg = (uint16_t*)wp;

    hipLaunchKernelGGL(bcd_fill_i32_kernel, dim3(1), dim3(64), 0, st, bad, (int64_t)1, 0);
    CDQ_LAUNCH_CHECK();
    hipLaunchKernelGGL(bcd_check_parts_kernel, dim3((unsigned)T), dim3(256), sizeof(uint32_t) * (size_t)((d_in + 31) / 32), st, parts, (int)d_in, bad);
    CDQ_LAUNCH_CHECK();
    int rc = gradient_launch(H, Wt, scale, zero, Q, d_out, d_in, group, G0, st);
    if (rc != CDQ_OK) return rc;
    rc = extract_diag_launch(H, d_in, hdiag, st);
    if (rc != CDQ_OK) return rc;
    // several columns per workgroup where the columns' state and at least three pair-table rows fit in LDS
    int cw = 0, nst = 0;
    if (d_in % 16 == 0 && 5 * d_in / 16 <= BCDM_NT * BCDM_MAXI && !single)        // a row is 5 d_in / 16 chunks of 16 bytes
        for (int c : {8, 4, 2}) {
            const size_t fixed = bcdm_lds_bytes(d_in, group, c, 0);
            if (fixed >= 160 * 1024) continue;
            const int64_t fit = (int64_t)((160 * 1024 - fixed) / (10 * (size_t)(d_in / 2)));
            if (fit < 3 || d_in > (int64_t)bcdm_xpt(c) * BCDM_NT) continue;
            cw = c;
            nst = fit > 6 ? 6 : (int)fit;
            break;
        }
    // the wide-layer kernel where nothing else applies, and where it shares a pass over the pairs among more columns than
    // the kernels with the columns' state in LDS would (measured: d_in = 4608, 2 columns there 363 ms, 8 here 205 ms;
    // d_in = 3072, 4 there 106 ms, 16 here 64 ms; d_in = 2048, 8 there 24.1 ms, 16 here 26.6 ms)
    const bool use_wide = !single_ok || (wide && wide_ok) || (!single && cw < 8 && cpw >= 3);
    if (use_wide) {
        uint32_t* t_ik = (uint32_t*)table;
        uint16_t* t_thr = (uint16_t*)(table + 4 * (size_t)n_items);
        hipLaunchKernelGGL(bcdm_pair_gather_kernel, dim3((unsigned)((n_items + 255) / 256)), dim3(256), 0, st, H, parts,
                           (const int32_t*)bad, d_in, n_items, t_ik, t_thr, pair_h2);
        CDQ_LAUNCH_CHECK();
        const int tc = (int)(trace_cap > 0x7fffffffLL ? 0x7fffffffLL : trace_cap);
        const size_t wlds = bcdw_lds_bytes(d_in);
        const dim3 grid((unsigned)((d_out + cpw - 1) / cpw));
#define BCDW_CASE(B, C)                                                                                                          \
    if (bits == B && wcw == C) {                                                                                                 \
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(bcd2_wide_kernel<B, C>), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                (int)wlds) != hipSuccess)                                                                        \
            return CDQ_EHIP;                                                                                                     \
        hipLaunchKernelGGL((bcd2_wide_kernel<B, C>), grid, dim3(BCDW_NT), wlds, st, H, (const float*)hdiag, G0, Vg, scale, Q,    \
                           (const uint32_t*)t_ik, (const uint16_t*)t_thr, (const float*)pair_h2, (const int32_t*)bad, (int)d_out, \
                           (int)d_in, (int)group, (int)T, cpw, score_all ? 1 : 0, moves, G_out, trace, tc);                      \
        CDQ_LAUNCH_CHECK();                                                                                                      \
        return CDQ_OK;                                                                                                           \
    }
        BCDW_CASE(2, 16) BCDW_CASE(2, 8) BCDW_CASE(2, 4) BCDW_CASE(2, 2) BCDW_CASE(2, 1)
        BCDW_CASE(3, 16) BCDW_CASE(3, 8) BCDW_CASE(3, 4) BCDW_CASE(3, 2) BCDW_CASE(3, 1)
        BCDW_CASE(4, 16) BCDW_CASE(4, 8) BCDW_CASE(4, 4) BCDW_CASE(4, 2) BCDW_CASE(4, 1)
#undef BCDW_CASE
        return CDQ_EINVAL;
    }
    if (cw != 0) {
        hipLaunchKernelGGL(bcdm_pair_gather_kernel, dim3((unsigned)((n_items + 255) / 256)), dim3(256), 0, st, H, parts,
                           (const int32_t*)bad, d_in, n_items, (uint32_t*)pair_rec, (uint16_t*)((char*)pair_rec + 4 * n_items), pair_h2);
    } else {
        hipLaunchKernelGGL(bcd_pair_gather_kernel, dim3((unsigned)((n_items + 255) / 256)), dim3(256), 0, st, H, parts,
                           (const int32_t*)bad, d_in, n_items, pair_rec, pair_h2);
    }
    CDQ_LAUNCH_CHECK();
    if (cw != 0) {
        const size_t mlds = bcdm_lds_bytes(d_in, group, cw, nst);
        const int tc = (int)(trace_cap > 0x7fffffffLL ? 0x7fffffffLL : trace_cap);
        const dim3 grid((unsigned)((d_out + cw - 1) / cw));
#define BCDM_CASE(B, C)                                                                                                          \
    if (bits == B && cw == C) {                                                                                                  \
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(bcd2_multi_kernel<B, C>), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                (int)mlds) != hipSuccess)                                                                        \
            return CDQ_EHIP;                                                                                                     \
        hipLaunchKernelGGL((bcd2_multi_kernel<B, C>), grid, dim3(BCDM_NT), mlds, st, H, (const float*)hdiag, (const float*)G0,    \
                           scale, Q, (const uint32_t*)pair_rec, (const uint16_t*)((char*)pair_rec + 4 * n_items),                \
                           (const float*)pair_h2, (const int32_t*)bad, (int)d_out, (int)d_in,                                    \
                           (int)group, (int)T, nst, score_all ? 1 : 0, moves, G_out, trace, tc);                                 \
        CDQ_LAUNCH_CHECK();                                                                                                      \
        return CDQ_OK;                                                                                                           \
    }
        BCDM_CASE(2, 8) BCDM_CASE(2, 4) BCDM_CASE(2, 2)
        BCDM_CASE(3, 8) BCDM_CASE(3, 4) BCDM_CASE(3, 2)
        BCDM_CASE(4, 8) BCDM_CASE(4, 4) BCDM_CASE(4, 2)
#undef BCDM_CASE
        return CDQ_EINVAL;
    }
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
