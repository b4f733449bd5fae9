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

// Tile order for large matrices: workgroups are handed to the 8 XCDs round-robin, and each XCD has its own L2, so
// the 32 workgroups an XCD runs at a time should share operand column blocks.  Workgroup w belongs to XCD w % 8 and
// is that XCD's (w / 8)-th; consecutive runs of 32 of them form a patch of 4 x 8 tiles (12 column blocks for 32
// tiles instead of ~36 in row-major order).  Patches that lie wholly below the diagonal are not enumerated; tiles of
// a patch below the diagonal or outside the matrix return at once.  `rot` rotates the patch-to-XCD assignment
// (one value per token split) so that no XCD always gets the surplus patch.
constexpr int PATCH_R = 4, PATCH_C = 8;

__host__ __device__ inline int patch_row_first(int pi) { return (PATCH_R * pi) / PATCH_C; }     // first patch column reaching row block pi
__host__ __device__ inline int patch_count(int n_t) {
    const int PI = (n_t + PATCH_R - 1) / PATCH_R, PJ = (n_t + PATCH_C - 1) / PATCH_C;
    int c = 0;
    for (int pi = 0; pi < PI; ++pi) c += PJ - patch_row_first(pi);
    return c;
}
__device__ __forceinline__ bool tile_from_patch(int w, int rot, int n_t, int* I, int* J) {
    const int xcd = (w + rot) & 7, s = w >> 3;
    int p = (s >> 5) * 8 + xcd;
    const int pos = s & 31;
    const int PI = (n_t + PATCH_R - 1) / PATCH_R, PJ = (n_t + PATCH_C - 1) / PATCH_C;
    int pi = 0;
    for (; pi < PI; ++pi) {
        const int cnt = PJ - patch_row_first(pi);
        if (p < cnt) break;
        p -= cnt;
    }
    if (pi >= PI) return false;
    *I = PATCH_R * pi + (pos >> 3);
    *J = PATCH_C * (patch_row_first(pi) + p) + (pos & 7);
    return *I < n_t && *J < n_t && *J >= *I;
}

// ------------------------------------------------------------------------------------------ bf16
//
// 256 x 256 tile of H per workgroup of 4 wavefronts (one per SIMD), each wavefront 128 x 128 =
// 4 x 4 MFMA blocks with the 256 accumulator registers in AGPRs (a third less LDS traffic per FLOP
// than 128 x 64 on 8 wavefronts).  The token range is consumed in steps of 32; LDS is a ring of NSTAGE stages,
// each holding the two operand tiles of one step as 32 token rows of 256 columns (512 bytes).
// Loads run NSTAGE-1 steps ahead: a wavefront's direct global->LDS load moves 64 x 16 bytes = two
// token rows; lane l writes chunk position l%32 of row l/32 and fetches the global 16-byte chunk
// (l%32) ^ 4(row%4), i.e. the chunks of a row are XOR-swizzled by the row.  A transposing read by
// the 16 lanes j of a group fetches the 8-byte pieces (token tb + j/4, columns fb + 4(j%4) .. +3)
// and returns to lane j the tokens tb .. tb+3 of column fb + j; with the swizzle, the four token
// rows of a group fall into four different 64-byte bank groups, so reads and writes are
// conflict-free.  With a single wavefront per SIMD nothing else hides a stall, so the loop is a
// software pipeline over 16-token halves: the fragments of the next half are read while the MFMAs
// of the current one run (scheduling hints interleave one read behind each MFMA), the one barrier
// per step sits between the two halves, and issuing a step's loads costs a few scalar
// instructions (fixed per-lane offsets, a scalar base per step).  Tiles that stick out of the
// matrix, and a token range that is not a multiple of 32, take a plain path through registers
// with zero fill (same layout).

constexpr int T2 = 256;                 // tile of H: T2 x T2 per workgroup
constexpr int BK16 = 64;                // granularity of the token split (two steps)
constexpr int BKS = 32;                 // tokens per step
constexpr int ROWB = T2 * 2;            // LDS bytes per token row of a tile
constexpr int TILE_BYTES = BKS * ROWB;  // 16 KiB per operand per stage
constexpr int NSTAGE = 4;
constexpr int HESS_LDS = NSTAGE * 2 * TILE_BYTES;      // 128 KiB

typedef short s4v __attribute__((ext_vector_type(4)));
typedef short s8v __attribute__((ext_vector_type(8)));

// tokens tb..tb+3 (first read) and tb+4..tb+7 (second read) of this lane's column: the 8 contraction
// elements one lane feeds to v_mfma_f32_32x32x16_bf16
__device__ __forceinline__ bf8 read_frag(const char* p) {
    const s4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s4v*)(p));
    const s4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s4v*)(p + 4 * ROWB));
    const s8v both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf8, both);
}

// 16 bytes per lane from global memory straight into LDS at dst + 16 * lane (dst uniform over the wavefront).
// Written as assembly so that the waits stay ours: the compiler would make every LDS read wait for all
// direct loads in flight, the ones for later stages included.
__device__ __forceinline__ void lds_direct_load16(const void* src, const char* dst) {
    const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)dst);
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(src) : "m0", "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmem() {          // until at most N of this wavefront's vector-memory operations are pending
    if (N == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else if (N == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
    else if (N == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    else if (N == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else if (N == 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
}

__global__ __launch_bounds__(256) void hessian_bf16_kernel(const uint16_t* __restrict__ X, int64_t n, int64_t d_in,
                                                           int n_t, int64_t tokens_per_split,
                                                           float* __restrict__ out, int64_t split_stride, int patched) {
    extern __shared__ __attribute__((aligned(16))) char lds[];       // [NSTAGE][A tile | B tile]
    int I, J;
    if (patched) {
        if (!tile_from_patch((int)blockIdx.x, (int)blockIdx.z, n_t, &I, &J)) return;
    } else {
        tile_from_linear(blockIdx.x, n_t, &I, &J);
    }
    const bool diag = (I == J);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;           // 2 x 2 wavefronts, each 128 rows x 128 columns
    const int64_t i0 = (int64_t)I * T2, j0 = (int64_t)J * T2;
    const int64_t t_begin = (int64_t)blockIdx.z * tokens_per_split;
    const int64_t t_end = (t_begin + tokens_per_split < n) ? t_begin + tokens_per_split : n;
    const int n_steps = (int)((t_end - t_begin + BKS - 1) / BKS);

    f16v acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    // fragment read roles: 16-lane group g = lane/16 takes columns 16 (g%2) .. +15 of a 32-column fragment and the
    // token half g/2 of a 16-token sub-step; lane j of the group addresses token j/4, columns 4 (j%4) .. +3
    const int jj = lane & 15, gg = lane >> 4;
    const int rd_row = (8 * (gg >> 1) + (jj >> 2)) * ROWB + 8 * (jj & 1);
    const int rd_chunk = 2 * (gg & 1) + ((jj & 3) >> 1), rd_swz = jj & 12;
    int offA[4], offB[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) offA[b] = rd_row + (((wm * 16 + 4 * b + rd_chunk) ^ rd_swz) << 4);
#pragma unroll
    for (int b = 0; b < 4; ++b) offB[b] = rd_row + (((wn * 16 + 4 * b + rd_chunk) ^ rd_swz) << 4);

    // one wavefront per SIMD: the fragments of the next 16-token sub-step are fetched while the MFMAs of the
    // current one run (the matrix core works asynchronously to the wavefront's instruction stream)
    auto load_frags = [&](const char* At, const char* Bt, int ks, bf8 (&af)[4], bf8 (&bfr)[4]) {
        // in the order the MFMAs below want them: the first row block, all column blocks, the other row blocks
        af[0] = read_frag(At + offA[0] + ks * 16 * ROWB);
#pragma unroll
        for (int b = 0; b < 4; ++b) bfr[b] = read_frag(Bt + offB[b] + ks * 16 * ROWB);
#pragma unroll
        for (int b = 1; b < 4; ++b) af[b] = read_frag(At + offA[b] + ks * 16 * ROWB);
    };
    auto mfmas = [&](const bf8 (&af)[4], const bf8 (&bfr)[4]) {
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bfr[b], acc[a][b], 0, 0, 0);
    };
    auto interleave = [&]() {          // ask for one LDS read behind each MFMA instead of a block of reads, then a block of MFMAs
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
    };
    auto compute = [&](int stage) {    // plain form, for the path through registers
        const char* At = lds + stage * 2 * TILE_BYTES;
        const char* Bt = diag ? At : At + TILE_BYTES;
        static_assert(BKS == 32, "two sub-steps per step");
        bf8 a0[4], b0[4], a1[4], b1[4];
        load_frags(At, Bt, 0, a0, b0);
        load_frags(At, Bt, 1, a1, b1);
        mfmas(a0, b0);
        mfmas(a1, b1);
    };

    const bool interior = (i0 + T2 <= d_in) && (j0 + T2 <= d_in);
    if (n_steps <= 0) {
        // empty token range: the partial tile is zero
    } else if (interior && (t_end - t_begin) % BKS == 0) {
        // ---- direct global->LDS loads, NSTAGE-1 steps ahead.  A step's tiles are 32 (16 on the diagonal) loads of two
        // token rows each; wavefront w issues loads w, w+8, ... so every wavefront has the same number in flight.
        // Per load q the lane's byte offset from the first token row of the step is fixed; only a scalar base moves
        // from step to step, so issuing a step's loads costs a handful of scalar instructions.
        const int per_wave = diag ? 4 : 8;
        const int lrow = lane >> 5, lpos = lane & 31;
        uint32_t src_off[8];
        uint32_t dst_off[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int g = wave + 4 * q;                           // 0..15: A tile, 16..31: B tile
            const int op = g >> 4, row = 2 * (g & 15) + lrow;
            const int chunk = lpos ^ (4 * (row & 3));
            src_off[q] = (uint32_t)(((int64_t)row * d_in + (op ? j0 - i0 : 0) + 8 * chunk) * 2);
            dst_off[q] = (uint32_t)(op * TILE_BYTES + 2 * (g & 15) * ROWB);
        }
        const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)lds;
        const char* xbase = reinterpret_cast<const char*>(X + t_begin * d_in + i0);
        const int64_t step_bytes = (int64_t)BKS * d_in * 2;
        auto issue = [&](int step) {
            const char* base = xbase + (int64_t)step * step_bytes;
            const uint32_t stage_lds = lds_base + (uint32_t)((step % NSTAGE) * 2 * TILE_BYTES);
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                if (q < per_wave) {
                    const uint32_t m0v = __builtin_amdgcn_readfirstlane(stage_lds + dst_off[q]);
                    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(m0v), "v"(src_off[q]), "s"(base) : "m0", "memory");
                }
            }
        };
        // Software pipeline over half steps.  While the MFMAs of one 16-token half run, the fragments of the next half
        // are read; the barrier sits between the two halves of a step: behind it the next step's tiles are visible
        // (each wavefront has waited for its own loads) and the previous step's stage is free for new loads.
        auto wait_loads = [&](int groups_left) {          // until at most `groups_left` steps' worth of this wavefront's loads are pending
            if (diag) { if (groups_left >= 2) wait_vmem<8>(); else if (groups_left == 1) wait_vmem<4>(); else wait_vmem<0>(); }
            else      { if (groups_left >= 2) wait_vmem<16>(); else if (groups_left == 1) wait_vmem<8>(); else wait_vmem<0>(); }
        };
        static_assert(NSTAGE == 4, "the wait counts below assume three steps in flight");
        const int pro = n_steps < NSTAGE - 1 ? n_steps : NSTAGE - 1;
        for (int s0 = 0; s0 < pro; ++s0) issue(s0);
        wait_loads(pro - 1);
        __syncthreads();
        bf8 a0[4], b0[4], a1[4], b1[4];
        load_frags(lds, diag ? lds : lds + TILE_BYTES, 0, a0, b0);
        for (int step = 0; step + 1 < n_steps; ++step) {
            const char* At = lds + (step % NSTAGE) * 2 * TILE_BYTES;
            const char* Bt = diag ? At : At + TILE_BYTES;
            load_frags(At, Bt, 1, a1, b1);
            mfmas(a0, b0);
            interleave();
            const int in_flight = (n_steps - 1 - step < NSTAGE - 2) ? n_steps - 1 - step : NSTAGE - 2;   // steps step+1 .. already issued
            wait_loads(in_flight - 1);
            __syncthreads();
            if (step + NSTAGE - 1 < n_steps) issue(step + NSTAGE - 1);       // into the stage of step-1, which nobody reads any more
            const char* An = lds + ((step + 1) % NSTAGE) * 2 * TILE_BYTES;
            load_frags(An, diag ? An : An + TILE_BYTES, 0, a0, b0);
            mfmas(a1, b1);
            interleave();
        }
        {       // last step: nothing left to fetch behind it
            const char* At = lds + ((n_steps - 1) % NSTAGE) * 2 * TILE_BYTES;
            load_frags(At, diag ? At : At + TILE_BYTES, 1, a1, b1);
            mfmas(a0, b0);
            mfmas(a1, b1);
        }
    } else {
        // ---- edge tiles / ragged token range: through registers with zero fill, one stage, same layout
        const int cpos = tid & 31, rgrp = tid >> 5;                 // 8 row groups of 4 token rows, 32 chunks per row
        for (int step = 0; step < n_steps; ++step) {
            const int64_t t0 = t_begin + (int64_t)step * BKS;
            u4 r[2][4];
#pragma unroll
            for (int half = 0; half < 2; ++half)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int row = rgrp * 4 + q;
                    const int64_t t = t0 + row, col = (half ? j0 : i0) + 8 * (cpos ^ (4 * q));
                    r[half][q] = (u4){0u, 0u, 0u, 0u};
                    if (!(half && diag) && t < t_end && col < d_in) r[half][q] = *reinterpret_cast<const u4*>(X + t * d_in + col);
                }
            __syncthreads();                 // previous step's reads are done
#pragma unroll
            for (int half = 0; half < 2; ++half)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (!(half && diag))
                        *reinterpret_cast<u4*>(lds + half * TILE_BYTES + (rgrp * 4 + q) * ROWB + cpos * 16) = r[half][q];
            __syncthreads();
            compute(0);
        }
    }
    // 32x32 result block: lane l, element v -> row 8*(v/4) + 4*(l/32) + v%4, column l%32
    float* dst = out + (int64_t)blockIdx.z * split_stride;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = i0 + wm * 128 + a * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v & 3);
                const int64_t col = j0 + wn * 128 + b * 32 + (lane & 31);
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
                                                              hipFuncAttributeMaxDynamicSharedMemorySize, HESS_LDS);
        if (attr_rc != hipSuccess) return CDQ_EHIP;
        const bool patched = n_t >= 24;                  // enough tiles for every XCD to fill whole patches
        if (patched) grid.x = (unsigned)(8 * ((patch_count((int)n_t) + 7) / 8) * PATCH_R * PATCH_C);
        hipLaunchKernelGGL(hessian_bf16_kernel, grid, dim3(256), HESS_LDS, st, (const uint16_t*)X, n, d_in, (int)n_t, per, parts, stride,
                           patched ? 1 : 0);
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
