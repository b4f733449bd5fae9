// C = E * H for all output columns, E = scale*Q + zero - Wt formed on the fly, fp32 data with
// fp64 accumulation on the matrix cores (v_mfma_f64_16x16x4_f64).  Two epilogues:
//   gradient: G[j][k] = (float) C[j][k]            -- Algorithm 1, "Compute gradient" (weight space)
//   loss:     partial[item][j] = sum_k C[j][k]*E[j][k] over the item's columns -- Eq. (1) as e^T H e.
//             H is symmetric, so only the blocks on and above its diagonal are multiplied: with 128-wide
//             blocks, e^T H e = sum_cb ( 2 sum_{kb<cb} e[kb]^T H[kb,cb] e[cb] + e[cb]^T H[cb,cb] e[cb] ),
//             half the matrix-core work.  A work item is (128 columns j) x (column block cb) x (a chunk
//             of the contraction range [0, (cb+1)*128) that does not straddle the diagonal block's start);
//             the doubling is exact in fp64.  Chunks make the items of a small layer equally long.
// fp64 accumulation keeps the one rounding to fp32 reproducible: the result differs from a
// sequential fp64 sum only when that sum lies within ~1e-16 relative of a rounding boundary.
//
// Tile: 128 (columns j) x 128 (coordinates k) per workgroup of 16 wavefronts (4 x 4), each
// wavefront 32 x 32 = 2 x 2 MFMA blocks; contraction step 64, two LDS stages.  An fp64 MFMA occupies its SIMD
// for 64 cycles, so LDS bandwidth is irrelevant and the 4 wavefronts per SIMD are there to keep
// the matrix core fed across barriers and global-load latency.
#include "cdq_internal.h"

#include <mutex>

namespace cdq {

namespace {

typedef double d4 __attribute__((ext_vector_type(4)));

constexpr int BM = 128, BN = 128, BK = 64, LDP = 144;   // LDP % 32 == 16: the two k-rows read by lanes 0..31 hit disjoint banks
constexpr int NT = 1024;
constexpr int NP = BK / 32;          // 32-deep pieces of a step's tiles handled by each thread
constexpr size_t EH_LDS = 4 * sizeof(float) * BK * LDP + sizeof(double) * 4 * BM;

// residual of 4 consecutive coordinates of one column (zero outside the matrix)
template <bool VEC4>
__device__ __forceinline__ void residual4(const float* __restrict__ Wt, const uint8_t* __restrict__ Q,
                                          const float* __restrict__ scale, const float* __restrict__ zero,
                                          int64_t row, int64_t i0, int64_t d_out, int64_t d_in, int64_t group,
                                          int64_t n_grp, float out[4]) {
#pragma unroll
    for (int e = 0; e < 4; ++e) out[e] = 0.0f;
    if (row >= d_out || i0 >= d_in) return;
    const float* w = Wt + row * d_in + i0;
    const uint8_t* q = Q + row * d_in + i0;
    if (VEC4) {     // d_in % 4 == 0, group % 4 == 0, 16-byte aligned rows: the four share one group
        const int64_t gi = i0 / group;
        const float a = scale[row * n_grp + gi], b = zero[row * n_grp + gi];
        const float4 wv = *reinterpret_cast<const float4*>(w);
        const uint32_t qv = *reinterpret_cast<const uint32_t*>(q);
        out[0] = fmaf(a, (float)(qv & 0xffu), b) - wv.x;
        out[1] = fmaf(a, (float)((qv >> 8) & 0xffu), b) - wv.y;
        out[2] = fmaf(a, (float)((qv >> 16) & 0xffu), b) - wv.z;
        out[3] = fmaf(a, (float)(qv >> 24), b) - wv.w;
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (i0 + e < d_in) {
                const int64_t gi = (i0 + e) / group;
                out[e] = fmaf(scale[row * n_grp + gi], (float)q[e], zero[row * n_grp + gi]) - w[e];
            }
        }
    }
}

// MODE 0: the product (gradient).  MODE 1: the loss from the blocks of H on and above the diagonal.  MODE 2: the product
// and, from the same accumulators, each row's loss sum_k C_jk e_jk as one partial sum per (row, column block of H); blocks of
// rows can be switched off, and the rows can be sent elsewhere: row s of the operands goes to row row_map[s] of G, only
// rows below *n_rows_dev exist.
template <int MODE, bool VEC4>
__global__ __launch_bounds__(NT) void eh_gemm_kernel(const float* __restrict__ H, const float* __restrict__ Wt,
                                                     const float* __restrict__ scale, const float* __restrict__ zero,
                                                     const uint8_t* __restrict__ Q, int64_t d_out, int64_t d_in,
                                                     int64_t group, float* __restrict__ G,
                                                     double* __restrict__ partial, int chunk_blocks,
                                                     double* __restrict__ G64, const uint8_t* __restrict__ row_block_active,
                                                     const int32_t* __restrict__ row_map, const int32_t* __restrict__ n_rows_dev) {
    constexpr bool LOSS = MODE == 1;
    // two stages of As[k][m] = E[m0+m][k0+k] and Bs[k][n] = H[k0+k][n0+n]: the next step's tiles are written
    // while the current ones are multiplied, one barrier per step
    extern __shared__ __attribute__((aligned(16))) char eh_smem[];
    float (*As)[BK][LDP] = reinterpret_cast<float (*)[BK][LDP]>(eh_smem);
    float (*Bs)[BK][LDP] = reinterpret_cast<float (*)[BK][LDP]>(eh_smem + 2 * sizeof(float) * BK * LDP);
    double (*red)[BM] = reinterpret_cast<double (*)[BM]>(eh_smem + 4 * sizeof(float) * BK * LDP);

    // loss: the caller may only want some blocks of BM rows (the partial sums of the others are left as they are)
    if (LOSS && row_block_active != nullptr && row_block_active[blockIdx.x] == 0) return;
    if (MODE == 2 && row_block_active != nullptr && row_block_active[blockIdx.y] == 0) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3;
    // loss: consecutive workgroups take the same item for consecutive column tiles (they share the H blocks, and the
    // longest items of all column tiles start first); gradient: x = column block of H, y = column tile
    const int64_t m0 = (int64_t)(LOSS ? blockIdx.x : blockIdx.y) * BM;
    const int64_t n_grp = d_in / group;
    // gradient: item = column block, whole contraction range.  loss: decode (column block, chunk) from the item index;
    // column blocks are laid out from the last (longest range) to the first
    int64_t n0 = (int64_t)blockIdx.x * BN, k_begin = 0, k_end = d_in;
    bool has_diag = false;
    if (LOSS) {
        const int n_cb = (int)((d_in + BN - 1) / BN);
        int item = (int)blockIdx.y, cb = n_cb - 1;
        while (true) {
            const int items_cb = (cb + chunk_blocks) / chunk_blocks;        // ceil((cb + 1) / chunk_blocks)
            if (item < items_cb) break;
            item -= items_cb;
            --cb;
        }
        n0 = (int64_t)cb * BN;
        k_begin = (int64_t)item * chunk_blocks * BN;
        k_end = k_begin + (int64_t)chunk_blocks * BN;
        if (k_end >= n0 + BN) { k_end = n0 + BN; has_diag = true; }
        if (k_end > d_in) k_end = d_in;
    }

    d4 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = (d4){0.0, 0.0, 0.0, 0.0};

    // loader roles, per 32-deep piece of the step: one 4-wide run of the E tile (128 rows x 8 runs) and one of the
    // H tile (32 rows x 32 runs) per thread
    const int a_row = tid >> 3, a_k = (tid & 7) * 4;
    const int b_row = tid >> 5, b_col = (tid & 31) * 4;

    // The loads of a step are issued before the MFMAs of the previous one and only consumed after them: the raw
    // weights, codes and grid entries stay in registers, and the residual e = fma(a, q, b) - w is formed when the
    // tile is written to LDS (forming it at load time would make every wavefront wait out the memory latency in
    // front of its MFMAs).
    float rw[NP][4], rs[NP][4], rz[NP][4], rb[NP][4];
    uint32_t rq[NP][4];
    bool e_valid[NP];
    auto load_tiles = [&](int64_t k0) {
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int64_t row = m0 + a_row, i0 = k0 + 32 * p + a_k;
            e_valid[p] = row < d_out && i0 < d_in;
            if (e_valid[p]) {
                const float* w = Wt + row * d_in + i0;
                const uint8_t* q = Q + row * d_in + i0;
                if (VEC4) {     // d_in % 4 == 0, group % 4 == 0, 16-byte aligned rows: the four share one group
                    const int64_t gi = i0 / group;
                    const float4 wv = *reinterpret_cast<const float4*>(w);
                    rq[p][0] = *reinterpret_cast<const uint32_t*>(q);
                    rs[p][0] = scale[row * n_grp + gi];
                    rz[p][0] = zero[row * n_grp + gi];
                    rw[p][0] = wv.x; rw[p][1] = wv.y; rw[p][2] = wv.z; rw[p][3] = wv.w;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const bool ok = i0 + e < d_in;
                        const int64_t gi = ok ? (i0 + e) / group : 0;
                        rw[p][e] = ok ? w[e] : 0.0f;
                        rq[p][e] = ok ? q[e] : 0u;
                        rs[p][e] = ok ? scale[row * n_grp + gi] : 0.0f;
                        rz[p][e] = ok ? zero[row * n_grp + gi] : 0.0f;
                    }
                }
            }
            const int64_t hr = k0 + 32 * p + b_row, c0 = n0 + b_col;
            if (VEC4) {
                float4 hv = make_float4(0.f, 0.f, 0.f, 0.f);
                if (hr < d_in && c0 < d_in) hv = *reinterpret_cast<const float4*>(H + hr * d_in + c0);
                rb[p][0] = hv.x; rb[p][1] = hv.y; rb[p][2] = hv.z; rb[p][3] = hv.w;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) rb[p][e] = (hr < d_in && c0 + e < d_in) ? H[hr * d_in + c0 + e] : 0.0f;
            }
        }
    };

    auto store_tiles = [&](int st) {
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            float ra[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if (e_valid[p]) {
                if (VEC4) {
                    ra[0] = fmaf(rs[p][0], (float)(rq[p][0] & 0xffu), rz[p][0]) - rw[p][0];
                    ra[1] = fmaf(rs[p][0], (float)((rq[p][0] >> 8) & 0xffu), rz[p][0]) - rw[p][1];
                    ra[2] = fmaf(rs[p][0], (float)((rq[p][0] >> 16) & 0xffu), rz[p][0]) - rw[p][2];
                    ra[3] = fmaf(rs[p][0], (float)(rq[p][0] >> 24), rz[p][0]) - rw[p][3];
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) ra[e] = fmaf(rs[p][e], (float)rq[p][e], rz[p][e]) - rw[p][e];    // zero outside the matrix
                }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) As[st][32 * p + a_k + e][a_row] = ra[e];
            *reinterpret_cast<float4*>(&Bs[st][32 * p + b_row][b_col]) = make_float4(rb[p][0], rb[p][1], rb[p][2], rb[p][3]);
        }
    };
    load_tiles(k_begin);
    store_tiles(0);
    __syncthreads();
    int st = 0;
    for (int64_t k0 = k_begin; k0 < k_end; k0 += BK) {
        const bool more = k0 + BK < k_end;
        if (more) load_tiles(k0 + BK);
        if (LOSS && has_diag && k0 == n0 && k0 > k_begin) {      // what came from above the diagonal block counts twice
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = acc[i][j] * 2.0;
        }
#pragma unroll
        for (int ks = 0; ks < BK; ks += 4) {
            double a[2], b[2];
            const int kk = ks + (lane >> 4), mn = lane & 15;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                a[i] = (double)As[st][kk][wm * 32 + i * 16 + mn];
                b[i] = (double)Bs[st][kk][wn * 32 + i * 16 + mn];
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (more) store_tiles(st ^ 1);
        __syncthreads();
        st ^= 1;
    }

    // result layout of the 16x16 f64 block: lane l, element v  ->  row 4*v + l/16, column l%16
    const int r_in = lane >> 4, c_in = lane & 15;
    if (!LOSS) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int64_t row = m0 + wm * 32 + i * 16 + 4 * v + r_in;
                int64_t dst = row;
                bool live = row < d_out;
                if (MODE == 2 && row_map != nullptr) {
                    live = live && row < (int64_t)*n_rows_dev;
                    dst = live ? (int64_t)row_map[row] : 0;
                }
                if (live) {
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const int64_t col = n0 + wn * 32 + j * 16 + c_in;
                        if (col < d_in) {
                            if (G64 != nullptr) G64[dst * d_in + col] = acc[i][j][v];
                            else G[dst * d_in + col] = (float)acc[i][j][v];
                        }
                    }
                }
            }
    }
    if (MODE != 0 && (LOSS || partial != nullptr)) {
        // the residuals this lane's 16 sums meet, all fetched before the first is used (elements outside the matrix read
        // element (0, 0) and count as zero)
        float ev[2][4][2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int64_t row = m0 + wm * 32 + i * 16 + 4 * v + r_in;
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int64_t col = n0 + wn * 32 + j * 16 + c_in;
                    const bool ok = row < d_out && col < d_in;
                    const int64_t at = ok ? row * d_in + col : 0, ag = ok ? row * n_grp + col / group : 0;
                    const float e = fmaf(scale[ag], (float)Q[at], zero[ag]) - Wt[at];
                    ev[i][v][j] = ok ? e : 0.0f;
                }
            }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int lrow = wm * 32 + i * 16 + 4 * v + r_in;
                double s = 0.0;
#pragma unroll
                for (int j = 0; j < 2; ++j) s += acc[i][j][v] * (double)ev[i][v][j];
                // sum over the 16 lanes that share this row (fixed butterfly order)
                for (int o = 8; o; o >>= 1) s += __shfl_xor(s, o);
                if (c_in == 0) red[wn][lrow] = (!LOSS || has_diag) ? s : 2.0 * s;
            }
        __syncthreads();
        if (tid < BM) {
            const int64_t row = m0 + tid;
            if (row < d_out)
                partial[(int64_t)(LOSS ? blockIdx.y : blockIdx.x) * d_out + row] = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
        }
    }
}

// loss_per_col[j] = sum over the work items in index order; optional total over columns by one workgroup
__global__ __launch_bounds__(256) void loss_rows_kernel(const double* __restrict__ partial, int64_t d_out, int n_items,
                                                        double* __restrict__ row_loss) {
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= d_out) return;
    double s = 0.0;
    int t = 0;
    for (; t + 8 <= n_items; t += 8) {                                             // [item][column]: coalesced; eight loads in flight,
        double v[8];                                                               // added in index order
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = partial[(int64_t)(t + u) * d_out + j];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; t < n_items; ++t) s += partial[(int64_t)t * d_out + j];
    row_loss[j] = s;
}

// Work items of the loss per 128 columns j: the contraction range of column block cb, (cb+1) blocks, in chunks of
// `chunk` blocks.  Large layers take whole ranges (chunk = number of blocks); small ones are cut until there are
// enough items of equal length to fill the chip a few times over.
void loss_items(int64_t d_out, int64_t d_in, int* chunk, int64_t* n_items) {
    const int64_t n_cb = (d_in + BN - 1) / BN, gy = (d_out + BM - 1) / BM;
    auto count = [&](int64_t ch) {
        int64_t n = 0;
        for (int64_t cb = 0; cb < n_cb; ++cb) n += (cb + ch) / ch;
        return n;
    };
    int64_t ch = n_cb > 0 ? n_cb : 1;
    while (ch > 2 && count(ch) * gy < 4 * 256) ch = (ch + 1) / 2;
    *chunk = (int)ch;
    *n_items = count(ch);
}

__global__ __launch_bounds__(1024) void loss_total_kernel(const double* __restrict__ row_loss, int64_t d_out,
                                                          double* __restrict__ total) {
    __shared__ double sh[1024];
    double s = 0.0;
    for (int64_t j = threadIdx.x; j < d_out; j += 1024) s += row_loss[j];
    sh[threadIdx.x] = s;
    __syncthreads();
    for (int o = 512; o; o >>= 1) {
        if ((int)threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) total[0] = sh[0];
}

template <int MODE, bool VEC4>
bool eh_allow_lds() {
    static const hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void*>(eh_gemm_kernel<MODE, VEC4>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)EH_LDS);
    return rc == hipSuccess;
}

bool vec4_ok(const float* H, const float* Wt, const uint8_t* Q, int64_t d_in, int64_t group) {
    return d_in % 4 == 0 && group % 4 == 0 && ((uintptr_t)H & 15) == 0 && ((uintptr_t)Wt & 15) == 0 && ((uintptr_t)Q & 3) == 0;
}

}  // namespace

int loss_block_rows() { return BM; }

size_t loss_workspace_bytes(int64_t d_out, int64_t d_in) {
    int chunk;
    int64_t n_items;
    loss_items(d_out, d_in, &chunk, &n_items);
    return cdq_align_up((size_t)d_out * n_items * sizeof(double), 256) + cdq_align_up((size_t)d_out * sizeof(double), 256);
}

int gradient_launch(const float* H, const float* Wt, const float* scale, const float* zero, const uint8_t* Q,
                    int64_t d_out, int64_t d_in, int64_t group, float* G, hipStream_t st, double* G64) {
    if (d_out == 0) return CDQ_OK;
    const int64_t gx = (d_in + BN - 1) / BN, gy = (d_out + BM - 1) / BM;
    if (gy > 65535) return CDQ_EUNSUPPORTED;
    if (!eh_allow_lds<0, true>() || !eh_allow_lds<0, false>()) return CDQ_EHIP;
    if (vec4_ok(H, Wt, Q, d_in, group))
        hipLaunchKernelGGL((eh_gemm_kernel<0, true>), dim3((unsigned)gx, (unsigned)gy), dim3(NT), EH_LDS, st, H, Wt, scale, zero, Q,
                           d_out, d_in, group, G, (double*)nullptr, 0, G64, (const uint8_t*)nullptr, (const int32_t*)nullptr,
                           (const int32_t*)nullptr);
    else
        hipLaunchKernelGGL((eh_gemm_kernel<0, false>), dim3((unsigned)gx, (unsigned)gy), dim3(NT), EH_LDS, st, H, Wt, scale, zero, Q,
                           d_out, d_in, group, G, (double*)nullptr, 0, G64, (const uint8_t*)nullptr, (const int32_t*)nullptr,
                           (const int32_t*)nullptr);
    CDQ_LAUNCH_CHECK();
    return CDQ_OK;
}

// The product and, where loss_per_col is given, each row's loss from the same accumulators (ws as for loss_launch: one
// partial sum per row and column block of H).  row_block_active, row_map, n_rows_dev: see the kernel.
int gradient_loss_launch(const float* H, const float* Wt, const float* scale, const float* zero, const uint8_t* Q,
                         int64_t d_out, int64_t d_in, int64_t group, float* G, double* loss_per_col, void* ws, size_t ws_bytes,
                         hipStream_t st, const uint8_t* row_block_active, const int32_t* row_map, const int32_t* n_rows_dev) {
    if (d_out == 0) return CDQ_OK;
    const int64_t gx = (d_in + BN - 1) / BN, gy = (d_out + BM - 1) / BM;
    if (gy > 65535) return CDQ_EUNSUPPORTED;
    if ((row_map == nullptr) != (n_rows_dev == nullptr)) return CDQ_EINVAL;
    double* partial = nullptr;
    if (loss_per_col != nullptr) {          // the loss's own workspace holds at least one partial sum per row and column block
        if (ws == nullptr || ws_bytes < loss_workspace_bytes(d_out, d_in) || ((uintptr_t)ws & 255)) return CDQ_EWORKSPACE;
        partial = (double*)ws;
    }
    if (!eh_allow_lds<2, true>() || !eh_allow_lds<2, false>()) return CDQ_EHIP;
    if (vec4_ok(H, Wt, Q, d_in, group))
        hipLaunchKernelGGL((eh_gemm_kernel<2, true>), dim3((unsigned)gx, (unsigned)gy), dim3(NT), EH_LDS, st, H, Wt, scale, zero, Q,
                           d_out, d_in, group, G, partial, 0, (double*)nullptr, row_block_active, row_map, n_rows_dev);
    else
        hipLaunchKernelGGL((eh_gemm_kernel<2, false>), dim3((unsigned)gx, (unsigned)gy), dim3(NT), EH_LDS, st, H, Wt, scale, zero, Q,
                           d_out, d_in, group, G, partial, 0, (double*)nullptr, row_block_active, row_map, n_rows_dev);
    CDQ_LAUNCH_CHECK();
    if (loss_per_col != nullptr) {
        hipLaunchKernelGGL(loss_rows_kernel, dim3((unsigned)((d_out + 255) / 256)), dim3(256), 0, st, (const double*)partial, d_out, (int)gx,
                           loss_per_col);
        CDQ_LAUNCH_CHECK();
    }
    return CDQ_OK;
}

int loss_launch(const float* H, const float* Wt, const float* scale, const float* zero, const uint8_t* Q,
                int64_t d_out, int64_t d_in, int64_t group, double* loss_per_col, double* loss_total,
                void* ws, size_t ws_bytes, hipStream_t st, const uint8_t* row_block_active) {
    if (d_out == 0) {                 // empty layer: the total is an empty sum
        if (loss_total) {
            hipLaunchKernelGGL(loss_total_kernel, dim3(1), dim3(1024), 0, st, (const double*)nullptr, (int64_t)0, loss_total);
            CDQ_LAUNCH_CHECK();
        }
        return CDQ_OK;
    }
    if (ws == nullptr || ws_bytes < loss_workspace_bytes(d_out, d_in) || ((uintptr_t)ws & 255)) return CDQ_EWORKSPACE;
    const int64_t gy = (d_out + BM - 1) / BM;
    int chunk;
    int64_t gx;
    loss_items(d_out, d_in, &chunk, &gx);
    if (gx > 65535 || gy > 0x7fffffffLL) return CDQ_EUNSUPPORTED;
    double* partial = (double*)ws;
    double* rows_ws = (double*)((char*)ws + cdq_align_up((size_t)d_out * gx * sizeof(double), 256));
    double* rows = loss_per_col ? loss_per_col : rows_ws;
    if (!eh_allow_lds<1, true>() || !eh_allow_lds<1, false>()) return CDQ_EHIP;
    if (vec4_ok(H, Wt, Q, d_in, group))
        hipLaunchKernelGGL((eh_gemm_kernel<1, true>), dim3((unsigned)gy, (unsigned)gx), dim3(NT), EH_LDS, st, H, Wt, scale, zero, Q,
                           d_out, d_in, group, (float*)nullptr, partial, chunk, (double*)nullptr, row_block_active,
                           (const int32_t*)nullptr, (const int32_t*)nullptr);
    else
        hipLaunchKernelGGL((eh_gemm_kernel<1, false>), dim3((unsigned)gy, (unsigned)gx), dim3(NT), EH_LDS, st, H, Wt, scale, zero, Q,
                           d_out, d_in, group, (float*)nullptr, partial, chunk, (double*)nullptr, row_block_active,
                           (const int32_t*)nullptr, (const int32_t*)nullptr);
    CDQ_LAUNCH_CHECK();
    hipLaunchKernelGGL(loss_rows_kernel, dim3((unsigned)((d_out + 255) / 256)), dim3(256), 0, st, partial, d_out, (int)gx, rows);
    CDQ_LAUNCH_CHECK();
    if (loss_total) {
        hipLaunchKernelGGL(loss_total_kernel, dim3(1), dim3(1024), 0, st, rows, d_out, loss_total);
        CDQ_LAUNCH_CHECK();
    }
    return CDQ_OK;
}

// ---- the loss for callers that cannot allocate: the kernels above with their partial sums in a static device array

namespace {

constexpr size_t kLossScratchBytes = CDQ_LOSS_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char loss_scratch[kLossScratchBytes];

constexpr int kMaxDevices = 64;
void* loss_scratch_ptr[kMaxDevices];          // device address of this GPU's copy of the array, looked up once per device
std::mutex loss_scratch_mutex;

// The array's name is a host-side stand-in; the address the kernels can use comes from the runtime, per device.
int loss_scratch_of_current_device(void** out) {
    int dev = -1;
    CDQ_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return CDQ_EUNSUPPORTED;
    std::lock_guard<std::mutex> hold(loss_scratch_mutex);
    if (loss_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        CDQ_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(loss_scratch)));
        if (p == nullptr || ((uintptr_t)p & 255) != 0) return CDQ_EHIP;
        loss_scratch_ptr[dev] = p;
    }
    *out = loss_scratch_ptr[dev];
    return CDQ_OK;
}

}  // namespace

int loss_static_launch(const float* H, const float* Wt, const float* scale, const float* zero, const uint8_t* Q,
                       int64_t d_out, int64_t d_in, int64_t group, double* loss_per_col, double* loss_total, hipStream_t st) {
    if (loss_workspace_bytes(d_out, d_in) > kLossScratchBytes) return CDQ_EUNSUPPORTED;     // before anything touches the GPU
    void* scratch = nullptr;
    if (d_out > 0) {
        const int rc = loss_scratch_of_current_device(&scratch);
        if (rc != CDQ_OK) return rc;
    }
    // every partial sum the second kernel reads is written by the first one in the same call, so nothing has to be cleared
    return loss_launch(H, Wt, scale, zero, Q, d_out, d_in, group, loss_per_col, loss_total, scratch, kLossScratchBytes, st);
}

}  // namespace cdq
