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

constexpr int TB = 128;                 // tile of H per workgroup, fp32 path
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
//
// 256 x 256 tile of H per workgroup of 8 wavefronts (two per SIMD, so one can issue MFMAs while
// the other waits on LDS or the barrier), each wavefront 128 x 64 = 4 x 2 MFMA blocks, 64 tokens
// per step, LDS double-buffered (one barrier per step), next step's global loads in flight
// during the current step's MFMAs.
// LDS holds each operand tile transposed: 128 bytes (64 tokens) per column, the 16-byte token
// octets of a column XOR-swizzled with ((col >> 3) ^ col) & 7 so that both the transposing stores
// (8 consecutive lanes = 8 column octets) and the fragment reads (8 consecutive lanes = 8
// consecutive columns) touch 8 distinct bank groups.

constexpr int T2 = 256;                 // tile of H: T2 x T2 per workgroup
constexpr int BK16 = 64;                // tokens per step
constexpr int COLB = BK16 * 2;          // LDS bytes per column of the transposed tile
constexpr int TILE_BYTES = T2 * COLB;   // 32 KiB per operand per buffer

__device__ __forceinline__ int swz(int col, int octet) { return col * COLB + ((octet ^ (((col >> 3) ^ col) & 7)) << 4); }

// 8 tokens x 8 adjacent bf16 columns (16 bytes per token)
__device__ __forceinline__ void load_oct8(const uint16_t* __restrict__ X, int64_t t_end, int64_t d_in, int64_t t0,
                                          int64_t col, u4 w[8]) {
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const int64_t t = t0 + r;
        if (t < t_end && col < d_in) w[r] = *reinterpret_cast<const u4*>(X + t * d_in + col);
        else w[r] = (u4){0u, 0u, 0u, 0u};
    }
}
// transpose the 8x8 block in registers and store one 8-token run (16 bytes) per column
__device__ __forceinline__ void store_oct8(char* tile, int col_octet, int tok_octet, const u4 w[8]) {
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        u4 o;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t x = w[2 * k][c >> 1], y = w[2 * k + 1][c >> 1];
            o[k] = (c & 1) ? ((x >> 16) | (y & 0xffff0000u)) : ((x & 0xffffu) | (y << 16));
        }
        *reinterpret_cast<u4*>(tile + swz(col_octet * 8 + c, tok_octet)) = o;
    }
}

__global__ __launch_bounds__(512) void hessian_bf16_kernel(const uint16_t* __restrict__ X, int64_t n, int64_t d_in,
                                                           int n_t, int64_t tokens_per_split,
                                                           float* __restrict__ out, int64_t split_stride) {
    extern __shared__ __attribute__((aligned(16))) char lds[];       // [2 buffers][A tile | B tile]
    int I, J;
    tile_from_linear(blockIdx.x, n_t, &I, &J);
    const bool diag = (I == J);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3;           // 2 x 4 wavefronts, each 128 rows x 64 columns
    const int64_t i0 = (int64_t)I * T2, j0 = (int64_t)J * T2;
    const int64_t t_begin = (int64_t)blockIdx.z * tokens_per_split;
    const int64_t t_end = (t_begin + tokens_per_split < n) ? t_begin + tokens_per_split : n;

    f16v acc[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    // staging roles: threads 0..255 move the A tile (columns of block I), 256..511 the B tile
    const int half = tid >> 8;
    const int co = tid & 31, to = (tid >> 5) & 7;      // column octet, token octet
    const int64_t c0 = (half ? j0 : i0) + co * 8;
    const bool active = !(half && diag);               // a diagonal tile needs one operand only
    const bool interior = (i0 + T2 <= d_in) && (j0 + T2 <= d_in);
    u4 r[8];
    auto gload = [&](int64_t t0, bool full) {
        if (!active) return;
        if (full && interior) {                        // no bounds checks on the common path
            const uint16_t* p = X + (t0 + to * 8) * d_in + c0;
#pragma unroll
            for (int q = 0; q < 8; ++q) r[q] = *reinterpret_cast<const u4*>(p + q * d_in);
        } else {
            load_oct8(X, t_end, d_in, t0 + to * 8, c0, r);
        }
    };
    auto lstore = [&](int buf) {
        if (active) store_oct8(lds + buf * 2 * TILE_BYTES + half * TILE_BYTES, co, to, r);
    };

    if (t_begin < t_end) {
        gload(t_begin, t_begin + BK16 <= t_end);
        lstore(0);
    }
    __syncthreads();
    int buf = 0;
    for (int64_t t0 = t_begin; t0 < t_end; t0 += BK16) {
        const bool more = t0 + BK16 < t_end;
        if (more) gload(t0 + BK16, t0 + 2 * BK16 <= t_end);
        const char* At = lds + buf * 2 * TILE_BYTES;
        const char* Bt = diag ? At : At + TILE_BYTES;
#pragma unroll
        for (int ks = 0; ks < BK16 / 16; ++ks) {
            bf8 af[4], bfr[2];
            const int oct = ks * 2 + (lane >> 5);
#pragma unroll
            for (int b = 0; b < 4; ++b) af[b] = *reinterpret_cast<const bf8*>(At + swz(wm * 128 + b * 32 + (lane & 31), oct));
#pragma unroll
            for (int b = 0; b < 2; ++b) bfr[b] = *reinterpret_cast<const bf8*>(Bt + swz(wn * 64 + b * 32 + (lane & 31), oct));
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bfr[b], acc[a][b], 0, 0, 0);
        }
        if (more) lstore(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }
    // 32x32 result block: lane l, element v -> row 8*(v/4) + 4*(l/32) + v%4, column l%32
    float* dst = out + (int64_t)blockIdx.z * split_stride;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = i0 + wm * 128 + a * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v & 3);
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

// One workgroup per 32x32 block on or above the diagonal (2-D grid, blocks below it exit): sum the splits (ascending), add the
// previous H if accumulating, write the block and its mirror image (through LDS, so both
// writes are coalesced).  `parts` may alias H when there is a single split and no accumulation.
__global__ __launch_bounds__(256) void hessian_finalize_kernel(const float* parts, int splits, int64_t split_stride,
                                                               float* H, int64_t d_in, int nb, int accumulate) {
    __shared__ float tile[32][33];
    const int I = blockIdx.y, J = blockIdx.x;
    if (I > J) return;                                    // blocks below the diagonal are written as mirrors
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

int choose_splits(int64_t n, int64_t d_in, int bk, int tile) {
    const int64_t n_t = (d_in + tile - 1) / tile;
    const int64_t tiles = n_t * (n_t + 1) / 2;
    const int64_t max_splits = n / ((int64_t)bk * 16) > 0 ? n / ((int64_t)bk * 16) : 1;   // >= 16 steps per split
    int64_t splits = 1;
    if (tile == TB) {                     // small fp32 tiles, several workgroups per CU: just fill the chip twice
        while (tiles * splits < 512 && splits < 32) splits *= 2;
    } else if (tiles <= 256) {            // one workgroup per CU: fill exactly one round
        splits = 256 / tiles;
    } else {                              // few rounds: pick the split count that wastes least of the last round
        double best = 0.0;
        for (int64_t sp = 1; sp <= 4; ++sp) {
            const double rounds = (double)(tiles * sp) / 256.0;
            const double eff = rounds / (double)((tiles * sp + 255) / 256);
            if (eff > best + 0.03) { best = eff; splits = sp; }
            if (best >= 0.9) break;
        }
    }
    if (splits > max_splits) splits = max_splits;
    if (splits > 32) splits = 32;
    if (splits < 1) splits = 1;
    return (int)splits;
}

}  // namespace

size_t hessian_workspace_bytes(int64_t n, int64_t d_in) {
    const int s32 = choose_splits(n, d_in, BK32, TB), s16 = choose_splits(n, d_in, BK16, T2);
    const int splits = s32 > s16 ? s32 : s16;          // the dtype is not known here: cover both paths
    return cdq_align_up((size_t)splits * d_in * d_in * sizeof(float), 256) + 256;
}

int hessian_launch(const void* X, int x_dtype, int64_t n, int64_t d_in, float* H, int accumulate, float lambda_rel,
                   void* ws, size_t ws_bytes, hipStream_t st) {
    const int bk = (x_dtype == CDQ_BF16) ? BK16 : BK32;
    const int tile = (x_dtype == CDQ_BF16) ? T2 : TB;
    int splits = choose_splits(n, d_in, bk, tile);
    const int64_t n_t = (d_in + tile - 1) / tile;
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
    if (x_dtype == CDQ_BF16) {
        static const hipError_t attr_rc = hipFuncSetAttribute(reinterpret_cast<const void*>(hessian_bf16_kernel),
                                                              hipFuncAttributeMaxDynamicSharedMemorySize, 4 * TILE_BYTES);
        if (attr_rc != hipSuccess) return CDQ_EHIP;
        hipLaunchKernelGGL(hessian_bf16_kernel, grid, dim3(512), 4 * TILE_BYTES, st, (const uint16_t*)X, n, d_in, (int)n_t, per, parts, stride);
    }
    else
        hipLaunchKernelGGL(hessian_f32_kernel, grid, dim3(256), 0, st, (const float*)X, n, d_in, (int)n_t, per, parts, stride);
    CDQ_LAUNCH_CHECK();
    const int64_t nb = (d_in + 31) / 32;
    if (nb > 65535) return CDQ_EUNSUPPORTED;
    hipLaunchKernelGGL(hessian_finalize_kernel, dim3((unsigned)nb, (unsigned)nb), dim3(256), 0, st, parts, splits, stride, H, d_in,
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
