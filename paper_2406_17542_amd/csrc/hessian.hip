// H = X^T X (paper Section 3, Notation; Algorithm 1 "Compute Hessian") on the matrix cores.
//
// X is [n][d_in] row-major and the contraction runs over the n tokens, so both MFMA operands
// are read "down the columns" of X.  bf16 path: v_mfma_f32_32x32x16_bf16 wants, per lane, 8
// consecutive tokens of one column; tiles of X are therefore transposed on their way into LDS
// (each lane loads one 32-bit column pair for 8 tokens, regroups the 16-bit halves in
// registers and stores one 16-byte token run per column).  fp32 path: v_mfma_f32_32x32x2_f32
// takes one element per lane, no transposition needed.
//
// Only tiles on or above the diagonal are computed (H is symmetric); the token range may be
// split over grid.z, each split writing its partial tile; a second kernel sums the splits in a
// fixed order (so results are reproducible), optionally adds the previous H (streaming over
// token chunks), and mirrors into the lower triangle.
#include "cdq_internal.h"

namespace cdq {

namespace {

typedef float f16v __attribute__((ext_vector_type(16)));
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

constexpr int TB = 128;                 // tile of H: TB x TB per workgroup
constexpr int BK16 = 64;                // tokens per step, bf16 path
constexpr int ROWB = BK16 * 2 + 16;     // LDS bytes per column of the transposed tile (padded)
constexpr int BK32 = 16;                // tokens per step, fp32 path
constexpr int LDF = TB + 16;            // LDS floats per token row, fp32 path (LDF % 32 == 16)

__device__ __forceinline__ void tile_from_linear(int lin, int n_t, int* I, int* J) {
    // enumerate pairs I <= J row by row: row I holds n_t - I tiles
    int i = 0, rem = lin;
    while (rem >= n_t - i) { rem -= n_t - i; ++i; }
    *I = i;
    *J = i + rem;
}

// ------------------------------------------------------------------------------------------ bf16

// 8 tokens x 1 column pair (two adjacent bf16 columns as one 32-bit word per token)
__device__ __forceinline__ void load_pair8(const uint16_t* __restrict__ X, int64_t n, int64_t d_in, int64_t t0,
                                           int64_t col, uint32_t w[8]) {
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const int64_t t = t0 + r;
        w[r] = (t < n && col < d_in) ? *reinterpret_cast<const uint32_t*>(X + t * d_in + col) : 0u;
    }
}
__device__ __forceinline__ void store_pair8(char* tile, int colpair, int tgroup, const uint32_t w[8]) {
    u4 lo, hi;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        lo[k] = (w[2 * k] & 0xffffu) | (w[2 * k + 1] << 16);
        hi[k] = (w[2 * k] >> 16) | (w[2 * k + 1] & 0xffff0000u);
    }
    *reinterpret_cast<u4*>(tile + (2 * colpair) * ROWB + tgroup * 16) = lo;
    *reinterpret_cast<u4*>(tile + (2 * colpair + 1) * ROWB + tgroup * 16) = hi;
}

__global__ __launch_bounds__(256) void hessian_bf16_kernel(const uint16_t* __restrict__ X, int64_t n, int64_t d_in,
                                                           int n_t, int64_t tokens_per_split,
                                                           float* __restrict__ out, int64_t split_stride) {
    __shared__ __attribute__((aligned(16))) char As[TB * ROWB];
    __shared__ __attribute__((aligned(16))) char Bs[TB * ROWB];
    int I, J;
    tile_from_linear(blockIdx.x, n_t, &I, &J);
    const bool diag = (I == J);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t i0 = (int64_t)I * TB, j0 = (int64_t)J * TB;
    const int64_t t_begin = (int64_t)blockIdx.z * tokens_per_split;
    const int64_t t_end = (t_begin + tokens_per_split < n) ? t_begin + tokens_per_split : n;

    f16v acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    const int cp = tid & 63, tg = tid >> 6;          // column pair, token group (and tg + 4)
    uint32_t ra0[8], ra1[8], rb0[8], rb1[8];
    auto gload = [&](int64_t t0) {
        load_pair8(X, t_end, d_in, t0 + tg * 8, i0 + 2 * cp, ra0);
        load_pair8(X, t_end, d_in, t0 + (tg + 4) * 8, i0 + 2 * cp, ra1);
        if (!diag) {
            load_pair8(X, t_end, d_in, t0 + tg * 8, j0 + 2 * cp, rb0);
            load_pair8(X, t_end, d_in, t0 + (tg + 4) * 8, j0 + 2 * cp, rb1);
        }
    };

    if (t_begin < t_end) gload(t_begin);
    for (int64_t t0 = t_begin; t0 < t_end; t0 += BK16) {
        __syncthreads();
        store_pair8(As, cp, tg, ra0);
        store_pair8(As, cp, tg + 4, ra1);
        if (!diag) {
            store_pair8(Bs, cp, tg, rb0);
            store_pair8(Bs, cp, tg + 4, rb1);
        }
        __syncthreads();
        if (t0 + BK16 < t_end) gload(t0 + BK16);
        const char* Bsrc = diag ? As : Bs;
#pragma unroll
        for (int ks = 0; ks < BK16 / 16; ++ks) {
            bf8 af[2], bfr[2];
            const int koff = ks * 32 + (lane >> 5) * 16;
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                af[b] = *reinterpret_cast<const bf8*>(As + (wm * 64 + b * 32 + (lane & 31)) * ROWB + koff);
                bfr[b] = *reinterpret_cast<const bf8*>(Bsrc + (wn * 64 + b * 32 + (lane & 31)) * ROWB + koff);
            }
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bfr[b], acc[a][b], 0, 0, 0);
        }
    }
    // 32x32 result block: lane l, element v -> row 8*(v/4) + 4*(l/32) + v%4, column l%32
    float* dst = out + (int64_t)blockIdx.z * split_stride;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = i0 + wm * 64 + a * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v & 3);
                const int64_t col = j0 + wn * 64 + b * 32 + (lane & 31);
                if (row < d_in && col < d_in) dst[row * d_in + col] = acc[a][b][v];
            }
}

// ------------------------------------------------------------------------------------------ fp32

__global__ __launch_bounds__(256) void hessian_f32_kernel(const float* __restrict__ X, int64_t n, int64_t d_in, int n_t,
                                                          int64_t tokens_per_split, float* __restrict__ out,
                                                          int64_t split_stride) {
    __shared__ float As[BK32][LDF];
    __shared__ float Bs[BK32][LDF];
    int I, J;
    tile_from_linear(blockIdx.x, n_t, &I, &J);
    const bool diag = (I == J);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t i0 = (int64_t)I * TB, j0 = (int64_t)J * TB;
    const int64_t t_begin = (int64_t)blockIdx.z * tokens_per_split;
    const int64_t t_end = (t_begin + tokens_per_split < n) ? t_begin + tokens_per_split : n;

    f16v acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    const int lr = tid >> 4, lc = (tid & 15) * 8;     // 16 token rows x 16 threads x 8 columns
    float ra[8], rb[8];
    auto gload = [&](int64_t t0) {
        const int64_t t = t0 + lr;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int64_t ca = i0 + lc + e, cb = j0 + lc + e;
            ra[e] = (t < t_end && ca < d_in) ? X[t * d_in + ca] : 0.0f;
            rb[e] = (!diag && t < t_end && cb < d_in) ? X[t * d_in + cb] : 0.0f;
        }
    };
    if (t_begin < t_end) gload(t_begin);
    for (int64_t t0 = t_begin; t0 < t_end; t0 += BK32) {
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            As[lr][lc + e] = ra[e];
            if (!diag) Bs[lr][lc + e] = rb[e];
        }
        __syncthreads();
        if (t0 + BK32 < t_end) gload(t0 + BK32);
        const float(*Bsrc)[LDF] = diag ? As : Bs;
#pragma unroll
        for (int ks = 0; ks < BK32; ks += 2) {
            float af[2], bfr[2];
            const int kk = ks + (lane >> 5);
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                af[b] = As[kk][wm * 64 + b * 32 + (lane & 31)];
                bfr[b] = Bsrc[kk][wn * 64 + b * 32 + (lane & 31)];
            }
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[a], bfr[b], acc[a][b], 0, 0, 0);
        }
    }
    float* dst = out + (int64_t)blockIdx.z * split_stride;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = i0 + wm * 64 + a * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v & 3);
                const int64_t col = j0 + wn * 64 + b * 32 + (lane & 31);
                if (row < d_in && col < d_in) dst[row * d_in + col] = acc[a][b][v];
            }
}

// ------------------------------------------------------------------------------------------ finalize

// One workgroup per 32x32 block on or above the diagonal: sum the splits (ascending), add the
// previous H if accumulating, write the block and its mirror image (through LDS, so both
// writes are coalesced).  `parts` may alias H when there is a single split and no accumulation.
__global__ __launch_bounds__(256) void hessian_finalize_kernel(const float* parts, int splits, int64_t split_stride,
                                                               float* H, int64_t d_in, int nb, int accumulate) {
    __shared__ float tile[32][33];
    int I, J;
    tile_from_linear(blockIdx.x, nb, &I, &J);
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
    for (int r = ty; r < 32; r += 8) {
        const int64_t row = (int64_t)I * 32 + r, col = (int64_t)J * 32 + tx;
        float v = 0.0f;
        if (row < d_in && col < d_in) {
            // in diagonal blocks take the entry on or above the diagonal for both positions
            const int64_t rr = (I == J && row > col) ? col : row, cc = (I == J && row > col) ? row : col;
            for (int z = 0; z < splits; ++z) v += parts[z * split_stride + rr * d_in + cc];
            if (accumulate) v += H[rr * d_in + cc];
        }
        tile[r][tx] = v;
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        const int64_t row = (int64_t)I * 32 + r, col = (int64_t)J * 32 + tx;
        if (row < d_in && col < d_in) H[row * d_in + col] = tile[r][tx];
        if (I != J) {
            const int64_t mrow = (int64_t)J * 32 + r, mcol = (int64_t)I * 32 + tx;
            if (mrow < d_in && mcol < d_in) H[mrow * d_in + mcol] = tile[tx][r];
        }
    }
}

__global__ __launch_bounds__(1024) void diag_mean_kernel(const float* __restrict__ H, int64_t d_in, float* __restrict__ out) {
    __shared__ double sh[1024];
    double s = 0.0;
    for (int64_t i = threadIdx.x; i < d_in; i += 1024) s += (double)H[i * d_in + i];
    sh[threadIdx.x] = s;
    __syncthreads();
    for (int o = 512; o; o >>= 1) {
        if ((int)threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = (float)(sh[0] / (double)d_in);
}
__global__ __launch_bounds__(256) void add_damping_kernel(float* __restrict__ H, int64_t d_in, float lambda_rel,
                                                          const float* __restrict__ mean) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < d_in) H[i * d_in + i] += lambda_rel * mean[0];
}

int choose_splits(int64_t n, int64_t d_in, int bk) {
    const int64_t n_t = (d_in + TB - 1) / TB;
    const int64_t tiles = n_t * (n_t + 1) / 2;
    int splits = 1;
    // enough workgroups for two per CU, but keep at least 8 steps of tokens per split
    while (tiles * splits < 512 && splits < 32 && n / (splits * 2) >= (int64_t)bk * 8) splits *= 2;
    return splits;
}

}  // namespace

size_t hessian_workspace_bytes(int64_t n, int64_t d_in) {
    const int splits = choose_splits(n, d_in, BK32 /* the smaller step: never under-estimates */);
    return cdq_align_up((size_t)splits * d_in * d_in * sizeof(float), 256) + 256;
}

int hessian_launch(const void* X, int x_dtype, int64_t n, int64_t d_in, float* H, int accumulate, float lambda_rel,
                   void* ws, size_t ws_bytes, hipStream_t st) {
    const int bk = (x_dtype == CDQ_BF16) ? BK16 : BK32;
    int splits = choose_splits(n, d_in, bk);
    const int64_t n_t = (d_in + TB - 1) / TB;
    const int64_t tiles = n_t * (n_t + 1) / 2;
    if (tiles > 0x7fffffffLL) return CDQ_EUNSUPPORTED;
    const size_t part_bytes = cdq_align_up((size_t)splits * d_in * d_in * sizeof(float), 256);
    const bool in_place = (splits == 1 && !accumulate);
    const bool need_ws = !in_place || lambda_rel != 0.0f;
    if (need_ws && (ws == nullptr || ((uintptr_t)ws & 255) || ws_bytes < part_bytes + 256)) return CDQ_EWORKSPACE;
    float* parts = in_place ? H : (float*)ws;
    float* mean_slot = need_ws ? (float*)((char*)ws + part_bytes) : nullptr;
    int64_t per = (n + splits - 1) / splits;
    per = (per + bk - 1) / bk * bk;
    if (per == 0) per = bk;
    const int64_t stride = d_in * d_in;
    dim3 grid((unsigned)tiles, 1, (unsigned)splits);
    if (x_dtype == CDQ_BF16)
        hipLaunchKernelGGL(hessian_bf16_kernel, grid, dim3(256), 0, st, (const uint16_t*)X, n, d_in, (int)n_t, per, parts, stride);
    else
        hipLaunchKernelGGL(hessian_f32_kernel, grid, dim3(256), 0, st, (const float*)X, n, d_in, (int)n_t, per, parts, stride);
    CDQ_LAUNCH_CHECK();
    const int64_t nb = (d_in + 31) / 32;
    const int64_t fblocks = nb * (nb + 1) / 2;
    if (fblocks > 0x7fffffffLL) return CDQ_EUNSUPPORTED;
    hipLaunchKernelGGL(hessian_finalize_kernel, dim3((unsigned)fblocks), dim3(256), 0, st, parts, splits, stride, H, d_in,
                       (int)nb, accumulate);
    CDQ_LAUNCH_CHECK();
    if (lambda_rel != 0.0f) {
        hipLaunchKernelGGL(diag_mean_kernel, dim3(1), dim3(1024), 0, st, H, d_in, mean_slot);
        CDQ_LAUNCH_CHECK();
        hipLaunchKernelGGL(add_damping_kernel, dim3((unsigned)((d_in + 255) / 256)), dim3(256), 0, st, H, d_in, lambda_rel, mean_slot);
        CDQ_LAUNCH_CHECK();
    }
    return CDQ_OK;
}

}  // namespace cdq
