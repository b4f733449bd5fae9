// H = X^T X (paper Section 3, Notation; Algorithm 1 "Compute Hessian") on the matrix cores.
//
// X is [n][d_in] row-major and the contraction runs over the n tokens, so both MFMA operands
// are read "down the columns" of X.  bf16 path: v_mfma_f32_32x32x16_bf16 wants, per lane, 8
// tokens of one column.  Tiles of X are copied into LDS as they lie in memory (token rows) by
// gfx950's direct global->LDS loads, several steps ahead and without passing through registers,
// and the fragments are read with the transposing LDS load (ds_read_b64_tr_b16), which hands each
// lane four tokens of one column out of a 4-token x 16-column block addressed by 16 lanes.
// fp32 path: v_mfma_f32_32x32x2_f32 takes one element per lane, no transposition needed.
//
// Only tiles on or above the diagonal are computed (H is symmetric); the token range may be
// split over grid.z, each split writing its partial tile; a second kernel sums the splits in a
// fixed order (so results are reproducible), optionally adds the previous H (streaming over
// token chunks), and mirrors into the lower triangle.
#include "cdq_internal.h"
#include "tile256.h"

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

// Work distribution for large matrices (n_t >= kBalancedMinTiles tiles per side).  Workgroups are handed to the 8 XCDs
// round-robin (workgroup w runs on XCD w % 8) and each XCD has its own L2, so the 32 workgroups an XCD runs at a time
// should share operand column blocks.  The tiles on and above the diagonal are therefore listed patch by patch
// (PATCH_R x PATCH_C tiles: 12 column blocks for 32 tiles instead of ~36 in row-major order), and XCD x takes the
// x-th eighth of that list, 32 tiles -- one per CU -- at a time.  What is left of an XCD's share after its last whole
// round of 32 would keep a few CUs busy for a whole tile while the rest idle: those tiles are cut along the tokens
// into as many slices as it takes to occupy all 32 CUs, each slice writes a partial tile, and a small kernel adds the
// partial tiles in ascending order (so the result does not depend on timing).
constexpr int PATCH_R = 4, PATCH_C = 8;
constexpr int kBalancedMinTiles = 23;        // 276 tiles: the first size that does not fit one round of 256 CUs
constexpr int kCusPerXcd = 32, kXcds = 8;

__host__ __device__ inline int patch_row_first(int pi) { return (PATCH_R * pi) / PATCH_C; }     // first patch column reaching row block pi
__host__ __device__ inline int patch_valid(int pi, int pj, int n_t) {                           // tiles of the patch with I <= J < n_t
    int c = 0;
    for (int r = 0; r < PATCH_R; ++r) {
        const int I = PATCH_R * pi + r;
        if (I >= n_t) break;
        const int lo = I > PATCH_C * pj ? I : PATCH_C * pj;
        const int hi = PATCH_C * pj + PATCH_C < n_t ? PATCH_C * pj + PATCH_C : n_t;
        if (hi > lo) c += hi - lo;
    }
    return c;
}
// the L-th tile of the patch-by-patch list
__host__ __device__ inline void tile_from_list(int L, int n_t, int* I, int* J) {
    const int PI = (n_t + PATCH_R - 1) / PATCH_R, PJ = (n_t + PATCH_C - 1) / PATCH_C;
    for (int pi = 0; pi < PI; ++pi)
        for (int pj = patch_row_first(pi); pj < PJ; ++pj) {
            const int c = patch_valid(pi, pj, n_t);
            if (L >= c) { L -= c; continue; }
            for (int r = 0; r < PATCH_R; ++r) {
                const int i = PATCH_R * pi + r;
                const int lo = i > PATCH_C * pj ? i : PATCH_C * pj;
                const int hi = PATCH_C * pj + PATCH_C < n_t ? PATCH_C * pj + PATCH_C : n_t;
                const int cnt = hi > lo ? hi - lo : 0;
                if (L < cnt) { *I = i; *J = lo + L; return; }
                L -= cnt;
            }
        }
    *I = *J = 0;        // not reached for L < number of tiles
}
// XCD x's share of the list: tiles [first, first + count); `whole` of them run as whole tiles, the remaining `rest`
// are cut into `slices` token slices each
struct XcdShare { int first, count, whole, rest, slices; };
__host__ __device__ inline XcdShare xcd_share(int x, int tiles) {
    XcdShare sh;
    sh.first = (int)(((int64_t)tiles * x) / kXcds);
    sh.count = (int)(((int64_t)tiles * (x + 1)) / kXcds) - sh.first;
    sh.rest = sh.count % kCusPerXcd;
    sh.whole = sh.count - sh.rest;
    sh.slices = sh.rest ? kCusPerXcd / sh.rest : 1;
    return sh;
}

// ------------------------------------------------------------------------------------------ bf16
//
// 256 x 256 tile of H per workgroup of 4 wavefronts: the pipelined matrix-core loop of tile256.h with both operand tiles
// taken from X (rows = tokens).  Tiles that stick out of the matrix and token ranges that are not a multiple of 32 take a
// plain path through registers with zero fill (same LDS layout).

using tile256::T2;
using tile256::BKS;
using tile256::ROWB;
using tile256::TILE_BYTES;
constexpr int BK16 = 64;                // granularity of the token split (two steps)
constexpr int HESS_LDS = tile256::LDS_BYTES;           // 128 KiB

// tokens tb..tb+7 of this lane's column, as the plain path feeds them to the MFMA
__device__ __forceinline__ bf8 read_frag(const char* p) { return __builtin_bit_cast(bf8, tile256::read_frag(p)); }

// Edge tiles and ragged token ranges: through registers with zero fill, one stage, same LDS layout.
__device__ __forceinline__ void hessian_tile_plain(const uint16_t* __restrict__ X, int64_t d_in, int64_t i0, int64_t j0, bool diag,
                                                   int64_t t_begin, int64_t t_end, char* lds, f16v (&acc)[4][4]) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int jj = lane & 15, gg = lane >> 4;
    const int rd_row = (8 * (gg >> 1) + (jj >> 2)) * ROWB + 8 * (jj & 1);
    const int rd_chunk = 2 * (gg & 1) + ((jj & 3) >> 1), rd_swz = jj & 12;
    int offA[4], offB[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) offA[b] = rd_row + (((wm * 16 + 4 * b + rd_chunk) ^ rd_swz) << 4);
#pragma unroll
    for (int b = 0; b < 4; ++b) offB[b] = rd_row + (((wn * 16 + 4 * b + rd_chunk) ^ rd_swz) << 4);
    const int n_steps = (int)((t_end - t_begin + BKS - 1) / BKS);
    const int cpos = tid & 31, rgrp = tid >> 5;                 // 8 row groups of 4 token rows, 32 chunks per row
    const char* At = lds;
    const char* Bt = diag ? At : At + TILE_BYTES;
    for (int step = 0; step < n_steps; ++step) {
        const int64_t t0 = t_begin + (int64_t)step * BKS;
        u4 r[2][4];
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int row = rgrp * 4 + q;
                const int64_t t = t0 + row, col = (hf ? j0 : i0) + 8 * (cpos ^ (4 * q));
                r[hf][q] = (u4){0u, 0u, 0u, 0u};
                if (!(hf && diag) && t < t_end && col < d_in) r[hf][q] = *reinterpret_cast<const u4*>(X + t * d_in + col);
            }
        __syncthreads();                 // previous step's reads are done
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (!(hf && diag))
                    *reinterpret_cast<u4*>(lds + hf * TILE_BYTES + (rgrp * 4 + q) * ROWB + cpos * 16) = r[hf][q];
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf8 af[4], bfr[4];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                af[b] = read_frag(At + offA[b] + ks * 16 * ROWB);
                bfr[b] = read_frag(Bt + offB[b] + ks * 16 * ROWB);
            }
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bfr[b], acc[a][b], 0, 0, 0);
        }
    }
}

// 32x32 result block: lane l, element v -> row 8*(v/4) + 4*(l/32) + v%4, column l%32
__device__ __forceinline__ void hessian_tile_store(const f16v (&acc)[4][4], int64_t d_in, int64_t i0, int64_t j0, float* __restrict__ dst,
                                                   int64_t ld, bool add_old) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int col = wn * 128 + b * 32 + (lane & 31);
            // what dst holds is fetched for the whole 32x32 block before any of it is used (element by element the compiler
            // waits out one round trip per value); elements outside the matrix read the tile's first element instead
            float old[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) old[v] = 0.0f;
            if (add_old) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = wm * 128 + a * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v & 3);
                    const bool ok = i0 + row < d_in && j0 + col < d_in;
                    old[v] = dst[ok ? row * ld + col : 0];
                }
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = wm * 128 + a * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v & 3);
                if (i0 + row < d_in && j0 + col < d_in) dst[row * ld + col] = add_old ? acc[a][b][v] + old[v] : acc[a][b][v];
            }
        }
}

// The plain path as a function of its own (a call, not inlined): the compiler then places its 256 accumulators without
// regard to the pipelined loop's.
__device__ __attribute__((noinline)) void hessian_tile_slow(const uint16_t* __restrict__ X, int64_t d_in, int I, int J, int64_t t_begin,
                                                            int64_t t_end, float* __restrict__ dst, int64_t ld, bool add_old, char* lds) {
    const int64_t i0 = (int64_t)I * T2, j0 = (int64_t)J * T2;
    f16v acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;
    if (t_end > t_begin) hessian_tile_plain(X, d_in, i0, j0, I == J, t_begin, t_end, lds, acc);       // an empty range leaves the partial tile zero
    hessian_tile_store(acc, d_in, i0, j0, dst, ld, add_old);
}

// One work item: tile (I, J) over the tokens [t_begin, t_end).  `dst` points at the tile's first element in a matrix of
// leading dimension `ld` (H itself, a split's partial matrix, or a 256 x 256 slot).  `add_old`: add what dst holds
// (streaming over chunks of tokens).  The two paths are kept apart down to the store, so that the 256 accumulators of
// one never have to be reconciled with those of the other.
__device__ __forceinline__ void hessian_tile(const uint16_t* __restrict__ X, int64_t d_in, int I, int J, int64_t t_begin, int64_t t_end,
                                             float* __restrict__ dst, int64_t ld, bool add_old, char* lds) {
    const int64_t i0 = (int64_t)I * T2, j0 = (int64_t)J * T2;
    const bool interior = (i0 + T2 <= d_in) && (j0 + T2 <= d_in);
    const int64_t len = t_end - t_begin;
    if (interior && len > 0 && len % BKS == 0) {
        f16v acc[4][4];
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;
        // a tile on the diagonal is not special here: its column block is loaded into both operand tiles (there are n_t such
        // tiles among n_t (n_t + 1) / 2, and a second code path would double the registers the compiler has to place)
        const int n_steps = (int)(len / BKS);
        const char* rows = reinterpret_cast<const char*>(X + t_begin * d_in);
        tile256::pipelined<tile256::Bf16>(rows + i0 * 2, d_in * 2, nullptr, n_steps, rows + j0 * 2, d_in * 2, n_steps, lds, acc);
        hessian_tile_store(acc, d_in, i0, j0, dst, ld, add_old);
    } else {
        hessian_tile_slow(X, d_in, I, J, t_begin, t_end, dst, ld, add_old, lds);
    }
}

// Small matrices: one workgroup per (tile, token split); every split writes its partial matrix, the finalize kernel adds them.
__global__ __launch_bounds__(256) void hessian_bf16_kernel(const uint16_t* __restrict__ X, int64_t n, int64_t d_in,
                                                           int n_t, int64_t tokens_per_split,
                                                           float* __restrict__ out, int64_t split_stride) {
    extern __shared__ __attribute__((aligned(16))) char lds[];       // [NSTAGE][A tile | B tile]
    int I, J;
    tile_from_linear(blockIdx.x, n_t, &I, &J);
    const int64_t t_begin = (int64_t)blockIdx.z * tokens_per_split;
    const int64_t t_end = (t_begin + tokens_per_split < n) ? t_begin + tokens_per_split : n;
    hessian_tile(X, d_in, I, J, t_begin, t_end, out + (int64_t)blockIdx.z * split_stride + (int64_t)I * T2 * d_in + (int64_t)J * T2, d_in,
                 false, lds);
}

// Large matrices: workgroup w is the (w / 8)-th of XCD w % 8 and works through that XCD's share of the tile list (see the top
// of this file): whole tiles go straight into H (added to what is there when accumulating), slices of the share's last
// tiles go to their slot of `partial` ([8 XCDs][32 slots][256 x 256]).
__global__ __launch_bounds__(256) void hessian_bf16_balanced_kernel(const uint16_t* __restrict__ X, int64_t n, int64_t d_in, int n_t,
                                                                    int tiles, float* __restrict__ H, int accumulate,
                                                                    float* __restrict__ partial) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int x = blockIdx.x % kXcds, k = blockIdx.x / kXcds;
    const XcdShare sh = xcd_share(x, tiles);
    int I, J;
    if (k < sh.whole) {
        tile_from_list(sh.first + k, n_t, &I, &J);
        hessian_tile(X, d_in, I, J, 0, n, H + (int64_t)I * T2 * d_in + (int64_t)J * T2, d_in, accumulate != 0, lds);
        return;
    }
    const int e = k - sh.whole;                   // slice e % slices of the share's (e / slices)-th leftover tile
    if (e >= sh.rest * sh.slices) return;
    tile_from_list(sh.first + sh.whole + e / sh.slices, n_t, &I, &J);
    int64_t per = (n + sh.slices - 1) / sh.slices;
    per = (per + BK16 - 1) / BK16 * BK16;
    const int64_t t_begin = (int64_t)(e % sh.slices) * per;
    const int64_t t_end = t_begin + per < n ? t_begin + per : n;
    hessian_tile(X, d_in, I, J, t_begin, t_end, partial + ((int64_t)x * kCusPerXcd + e) * T2 * T2, T2, false, lds);
}

// The leftover tiles of every XCD's share: H tile = (previous H tile when accumulating) + the slices' partial tiles in
// ascending order.  Grid: (leftover tile, XCD, 64 blocks of 4 rows); 256 threads = the tile's columns.
__global__ __launch_bounds__(256) void hessian_add_slices_kernel(const float* __restrict__ partial, float* __restrict__ H, int64_t d_in, int n_t,
                                                                 int tiles, int accumulate) {
    const int x = blockIdx.y, r = blockIdx.x;
    const XcdShare sh = xcd_share(x, tiles);
    if (r >= sh.rest) return;
    int I, J;
    tile_from_list(sh.first + sh.whole + r, n_t, &I, &J);
    const float* src = partial + ((int64_t)x * kCusPerXcd + (int64_t)r * sh.slices) * T2 * T2;
    const int64_t i0 = (int64_t)I * T2, j0 = (int64_t)J * T2;
    const int col = threadIdx.x;
    if (j0 + col >= d_in) return;
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const int row = blockIdx.z * 4 + rr;
        if (i0 + row < d_in) {
            float* h = H + (i0 + row) * d_in + j0 + col;
            float v = accumulate ? *h : 0.0f;
            for (int z0 = 0; z0 < sh.slices; z0 += 8) {           // eight slices' loads in flight, added in ascending order
                float pv[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) pv[u] = src[((int64_t)(z0 + u < sh.slices ? z0 + u : z0) * T2 + row) * T2 + col];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (z0 + u < sh.slices) v += pv[u];
            }
            *h = v;
        }
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
            const float* src = parts + rr * d_in + cc;
            for (int z0 = 0; z0 < splits; z0 += 8) {           // eight splits' loads in flight, added in ascending order
                float pv[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) pv[u] = src[(int64_t)(z0 + u < splits ? z0 + u : z0) * split_stride];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (z0 + u < splits) v += pv[u];
            }
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

bool use_balanced(int x_dtype, int64_t d_in) { return x_dtype == CDQ_BF16 && (d_in + T2 - 1) / T2 >= kBalancedMinTiles; }
constexpr size_t kSliceSlotsBytes = (size_t)kXcds * kCusPerXcd * T2 * T2 * sizeof(float);      // 64 MiB

}  // namespace

size_t hessian_workspace_bytes(int64_t n, int64_t d_in) {
    // the dtype is not known here: cover both paths
    const int s32 = choose_splits(n, d_in, BK32, TB);
    size_t bytes = cdq_align_up((size_t)s32 * d_in * d_in * sizeof(float), 256);
    const size_t b16 = use_balanced(CDQ_BF16, d_in) ? kSliceSlotsBytes
                                                    : cdq_align_up((size_t)choose_splits(n, d_in, BK16, T2) * d_in * d_in * sizeof(float), 256);
    if (b16 > bytes) bytes = b16;
    return bytes + 256;
}

namespace {

int launch_damping(float* H, int64_t d_in, float lambda_rel, float* mean_slot, hipStream_t st) {
    hipLaunchKernelGGL(diag_mean_kernel, dim3(1), dim3(1024), 0, st, H, d_in, mean_slot);
    CDQ_LAUNCH_CHECK();
    hipLaunchKernelGGL(add_damping_kernel, dim3((unsigned)((d_in + 255) / 256)), dim3(256), 0, st, H, d_in, lambda_rel, mean_slot);
    CDQ_LAUNCH_CHECK();
    return CDQ_OK;
}

// bf16, at least kBalancedMinTiles tiles per side: whole tiles straight into H, the leftover tiles of every XCD's share in
// token slices through 64 MiB of workspace, then the mirror
int hessian_launch_balanced(const uint16_t* X, int64_t n, int64_t d_in, float* H, bool accumulate, float lambda_rel, void* ws,
                            size_t ws_bytes, hipStream_t st) {
    const int64_t n_t = (d_in + T2 - 1) / T2;
    const int64_t tiles64 = n_t * (n_t + 1) / 2;
    if (tiles64 > 0x3fffffffLL) return CDQ_EUNSUPPORTED;
    const int tiles = (int)tiles64;
    if (ws == nullptr || ((uintptr_t)ws & 255) || ws_bytes < kSliceSlotsBytes + 256) return CDQ_EWORKSPACE;
    float* partial = (float*)ws;
    float* mean_slot = (float*)((char*)ws + kSliceSlotsBytes);
    static const hipError_t attr_rc = hipFuncSetAttribute(reinterpret_cast<const void*>(hessian_bf16_balanced_kernel),
                                                          hipFuncAttributeMaxDynamicSharedMemorySize, HESS_LDS);
    if (attr_rc != hipSuccess) return CDQ_EHIP;
    int per_xcd = 0, max_rest = 0;
    for (int x = 0; x < kXcds; ++x) {
        const XcdShare sh = xcd_share(x, tiles);
        const int w = sh.whole + sh.rest * sh.slices;
        if (w > per_xcd) per_xcd = w;
        if (sh.rest > max_rest) max_rest = sh.rest;
    }
    hipLaunchKernelGGL(hessian_bf16_balanced_kernel, dim3((unsigned)(kXcds * per_xcd)), dim3(256), HESS_LDS, st, X, n, d_in, (int)n_t, tiles, H,
                       accumulate ? 1 : 0, partial);
    CDQ_LAUNCH_CHECK();
    if (max_rest > 0) {
        hipLaunchKernelGGL(hessian_add_slices_kernel, dim3((unsigned)max_rest, kXcds, T2 / 4), dim3(256), 0, st, partial, H, d_in, (int)n_t, tiles,
                           accumulate ? 1 : 0);
        CDQ_LAUNCH_CHECK();
    }
    const int64_t nb = (d_in + 31) / 32;
    if (nb > 65535) return CDQ_EUNSUPPORTED;
    // the upper triangle is complete: one split, in place, nothing to add -- the finalize kernel only mirrors
    hipLaunchKernelGGL(hessian_finalize_kernel, dim3((unsigned)nb, (unsigned)nb), dim3(256), 0, st, H, 1, d_in * d_in, H, d_in, (int)nb, 0);
    CDQ_LAUNCH_CHECK();
    if (lambda_rel != 0.0f) return launch_damping(H, d_in, lambda_rel, mean_slot, st);
    return CDQ_OK;
}

}  // namespace

int hessian_launch(const void* X, int x_dtype, int64_t n, int64_t d_in, float* H, int accumulate, float lambda_rel,
                   void* ws, size_t ws_bytes, hipStream_t st) {
    if (use_balanced(x_dtype, d_in)) return hessian_launch_balanced((const uint16_t*)X, n, d_in, H, accumulate != 0, lambda_rel, ws, ws_bytes, st);
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
                                                              hipFuncAttributeMaxDynamicSharedMemorySize, HESS_LDS);
        if (attr_rc != hipSuccess) return CDQ_EHIP;
        hipLaunchKernelGGL(hessian_bf16_kernel, grid, dim3(256), HESS_LDS, st, (const uint16_t*)X, n, d_in, (int)n_t, per, parts, stride);
    }
    else
        hipLaunchKernelGGL(hessian_f32_kernel, grid, dim3(256), 0, st, (const float*)X, n, d_in, (int)n_t, per, parts, stride);
    CDQ_LAUNCH_CHECK();
    const int64_t nb = (d_in + 31) / 32;
    if (nb > 65535) return CDQ_EUNSUPPORTED;
    hipLaunchKernelGGL(hessian_finalize_kernel, dim3((unsigned)nb, (unsigned)nb), dim3(256), 0, st, parts, splits, stride, H, d_in,
                       (int)nb, accumulate);
    CDQ_LAUNCH_CHECK();
    if (lambda_rel != 0.0f) return launch_damping(H, d_in, lambda_rel, mean_slot, st);
    return CDQ_OK;
}

}  // namespace cdq
