// A cheap look at every clipping strength of the OWC grid search (paper Section 3.1, "Initializing a, b, q"; Eq. (2)
// searched for the smallest loss of Eq. (1)) before the exact evaluation.
//
// The search itself stays what it is: per column the grid point with the smallest fp64 loss e^T H e, equal losses
// keeping the larger gamma.  But the fp64 evaluation of one grid point costs a d_out x d_in x d_in matrix product, and on
// real layers the best grid point beats the runner-up by half a percent at the median.  So every grid point is first
// evaluated in fp16 on the matrix cores (fp32 accumulation, ~10 times the fp64 kernel's rate).  To fit fp16's range the
// product is taken in normalised form: with d = sqrt(diag H), R = H / (d d^T) (entries in [-1, 1]) and f = e * d divided by
// its largest magnitude s, e^T H e = s^2 f^T R f.  Rounding f and R to 11 bits moves a column's loss by a few 1e-4
// relative at most (less when many coordinates carry it).  Only grid points whose screened loss is within the margin of
// the column's smallest screened loss -- between one and two per column on average -- can be the fp64 winner; those are
// evaluated exactly by the caller, rank by rank.
//
// Kernels here: R and f in fp16; C = F R on v_mfma_f32_32x32x16_f16 with the epilogue sum_c C[j][c] F[j][c] per row and
// column block; the sum over the column blocks; and the ranking of a column's grid points.
#include "cdq_internal.h"
#include "tile256.h"

namespace cdq {
namespace {

typedef float f16v __attribute__((ext_vector_type(16)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

constexpr int SB = 128;                 // smallest tile of C: SB rows of F by SB columns of R (the rows are padded to 2 SB)
constexpr int SK = 64;                  // contraction step
constexpr int SROW = SK * 2 + 16;       // LDS bytes per tile row (144: 16-byte aligned, rows 8 apart share banks)
// A tile of TB x TB of C per workgroup of (TB / 64)^2 wavefronts, 64 x 64 each: TB = 256 (16 wavefronts, 144 KiB of LDS)
// halves the operand traffic from L2 per FLOP (9.5 TB/s of tile loads with the 128 x 128 tile).

__global__ __launch_bounds__(256) void fill_words_kernel(uint32_t* __restrict__ p, int64_t n, uint32_t v) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}

// d[k] = sqrt(H_kk), rd[k] = 1 / d[k]
__global__ __launch_bounds__(256) void owc_diag_kernel(const float* __restrict__ H, int64_t d_in, float* __restrict__ d, float* __restrict__ rd) {
    const int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k >= d_in) return;
    const float v = sqrtf(H[k * d_in + k]);
    d[k] = v;
    rd[k] = __fdiv_rn(1.0f, v);
}

// R[c][k] = H[c][k] / (d[c] d[k]) in fp16; one workgroup per row
__global__ __launch_bounds__(256) void owc_corr_f16_kernel(const float* __restrict__ H, int64_t d_in, const float* __restrict__ rd,
                                                           _Float16* __restrict__ R) {
    const int64_t c = blockIdx.x;
    const float rc = rd[c];
    for (int64_t k = threadIdx.x; k < d_in; k += 256) R[c * d_in + k] = (_Float16)((H[c * d_in + k] * rc) * rd[k]);
}

// Eq. (2) at one clipping strength for a column, e = fma(a, q, lo) - w as the loss kernel forms it; f = e * d; the row is
// stored as f / s in fp16 with s = max |f| (1 when the residual is zero) and s^2 goes to row_scale2.  One workgroup per
// column; rows past d_out of the padded buffer stay zero.
__global__ __launch_bounds__(256) void owc_residual_f16_kernel(const float* __restrict__ Wt, int64_t d_in, int bits,
                                                               const float* __restrict__ lo_in, const float* __restrict__ hi_in,
                                                               float gamma, const float* __restrict__ d, _Float16* __restrict__ F,
                                                               float* __restrict__ row_scale2) {
    __shared__ float smax[4];
    const int64_t j = blockIdx.x;
    const float lo = lo_in[j], hi = hi_in[j];
    const float top = (float)((1 << bits) - 1);
    float a = __fdiv_rn(gamma * (hi - lo), top);
    if (!(a > 0.0f) || isinf(a)) a = 1.0f;
    const float* w = Wt + j * d_in;
    auto f_of = [&](int64_t k) {
        const float wk = w[k];
        const float q = fminf(fmaxf(rintf(__fdiv_rn(wk - lo, a)), 0.0f), top);
        return (fmaf(a, q, lo) - wk) * d[k];
    };
    float m = 0.0f;
    for (int64_t k = threadIdx.x; k < d_in; k += 256) m = fmaxf(m, fabsf(f_of(k)));
    for (int o = 32; o; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if ((threadIdx.x & 63) == 0) smax[threadIdx.x >> 6] = m;
    __syncthreads();
    m = fmaxf(fmaxf(smax[0], smax[1]), fmaxf(smax[2], smax[3]));
    const float s = (m > 0.0f && m < INFINITY) ? m : 1.0f;
    const float rs = __fdiv_rn(1.0f, s);
    if (threadIdx.x == 0) row_scale2[j] = s * s;
    _Float16* f = F + j * d_in;
    for (int64_t k = threadIdx.x; k < d_in; k += 256) f[k] = (_Float16)(f_of(k) * rs);
}

// The same rows for a 16-byte aligned Wt (d_in is a multiple of 128 here): four coordinates per lane and load, the first
// 8192 coordinates' f kept in registers between the pass that finds s and the pass that stores, the rest formed again.
// Every value is formed by the expressions of the kernel above, so the two kernels store the same bits.
__global__ __launch_bounds__(256) void owc_residual_f16_vec_kernel(const float* __restrict__ Wt, int64_t d_in, int bits,
                                                                   const float* __restrict__ lo_in, const float* __restrict__ hi_in,
                                                                   float gamma, const float* __restrict__ d, _Float16* __restrict__ F,
                                                                   float* __restrict__ row_scale2) {
    constexpr int KEEP = 8;
    __shared__ float smax[4];
    const int64_t j = blockIdx.x;
    const float lo = lo_in[j], hi = hi_in[j];
    const float top = (float)((1 << bits) - 1);
    float a = __fdiv_rn(gamma * (hi - lo), top);
    if (!(a > 0.0f) || isinf(a)) a = 1.0f;
    const float4* w4 = reinterpret_cast<const float4*>(Wt + j * d_in);
    const float4* d4 = reinterpret_cast<const float4*>(d);
    const int n4 = (int)(d_in >> 2);
    auto f_one = [&](float wk, float dk) {
        const float q = fminf(fmaxf(rintf(__fdiv_rn(wk - lo, a)), 0.0f), top);
        return (fmaf(a, q, lo) - wk) * dk;
    };
    auto f_of = [&](int c) {
        const float4 w = w4[c], dd = d4[c];
        return make_float4(f_one(w.x, dd.x), f_one(w.y, dd.y), f_one(w.z, dd.z), f_one(w.w, dd.w));
    };
    auto amax = [](float m, const float4& f) { return fmaxf(fmaxf(m, fabsf(f.x)), fmaxf(fabsf(f.y), fmaxf(fabsf(f.z), fabsf(f.w)))); };
    float4 kept[KEEP];
    float m = 0.0f;
#pragma unroll
    for (int i = 0; i < KEEP; ++i) {
        const int c = (int)threadIdx.x + 256 * i;
        kept[i] = c < n4 ? f_of(c) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        m = amax(m, kept[i]);
    }
    for (int c = (int)threadIdx.x + 256 * KEEP; c < n4; c += 256) m = amax(m, f_of(c));
    for (int o = 32; o; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if ((threadIdx.x & 63) == 0) smax[threadIdx.x >> 6] = m;
    __syncthreads();
    m = fmaxf(fmaxf(smax[0], smax[1]), fmaxf(smax[2], smax[3]));
    const float s = (m > 0.0f && m < INFINITY) ? m : 1.0f;
    const float rs = __fdiv_rn(1.0f, s);
    if (threadIdx.x == 0) row_scale2[j] = s * s;
    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
    h4* f = reinterpret_cast<h4*>(F + j * d_in);
    auto put = [&](int c, const float4& v) {
        h4 o;
        o.x = (_Float16)(v.x * rs), o.y = (_Float16)(v.y * rs), o.z = (_Float16)(v.z * rs), o.w = (_Float16)(v.w * rs);
        f[c] = o;
    };
#pragma unroll
    for (int i = 0; i < KEEP; ++i) {
        const int c = (int)threadIdx.x + 256 * i;
        if (c < n4) put(c, kept[i]);
    }
    for (int c = (int)threadIdx.x + 256 * KEEP; c < n4; c += 256) put(c, f_of(c));
}

// f^T R f over the blocks of R on and above the diagonal (R is symmetric: its row c is its column c, and the blocks below
// the diagonal repeat the ones above): for column block cb the contraction runs over k < TB (cb + 1); the diagonal block
// enters at half weight and the sum is doubled at the end.
// A wavefront owns BLK x BLK blocks of 32 x 32 of the tile; partial[cb * WPR + h][j] = sum over the 32 BLK columns c of
// part h of column block cb of C[j][c] F[j][c], WPR = TB / (32 BLK) wavefronts side by side.
// F [rows][d_in], rows a multiple of TB, d_in a multiple of TB.  grid (d_in / TB, rows / TB), longest column blocks first.
template <int TB, int BLK>
__global__ __launch_bounds__((TB / (32 * BLK)) * (TB / (32 * BLK)) * 64) void owc_screen_kernel(const _Float16* __restrict__ E,
                                                                                               const _Float16* __restrict__ R, int64_t rows,
                                                                                               int64_t d_in, float* __restrict__ partial) {
    constexpr int WT = 32 * BLK;                                                                 // a wavefront's rows and columns of the tile
    constexpr int WPR = TB / WT, SNT = WPR * WPR * 64, STILE = TB * SROW, CPT = TB * 8 / SNT;    // wavefronts per tile row, threads, chunks per thread
    extern __shared__ __attribute__((aligned(16))) char lds[];             // [2 stages][F tile | R tile]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int cb = (int)(gridDim.x - 1 - blockIdx.x);
    const int64_t c0 = (int64_t)cb * TB, j0 = (int64_t)blockIdx.y * TB;
    const int wr = (wave / WPR) * WT, wc = (wave % WPR) * WT;                 // this wavefront's part of the tile
    const int n_steps = (cb + 1) * (TB / SK), diag_step = cb * (TB / SK);     // steps before diag_step lie above the diagonal block

    // a thread moves CPT 16-byte chunks of each operand tile per step: chunk id = tid + SNT i -> row id / 8, chunk id % 8
    u4 ra[CPT], rb[CPT];
    auto load = [&](int step) {
        const int64_t k0 = (int64_t)step * SK;
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            const int id = tid + SNT * i, row = id >> 3, kc = id & 7;
            ra[i] = *reinterpret_cast<const u4*>(E + (j0 + row) * d_in + k0 + kc * 8);
            rb[i] = *reinterpret_cast<const u4*>(R + (c0 + row) * d_in + k0 + kc * 8);
        }
    };
    // halve: the steps of the diagonal block enter with F / 2 (the epilogue doubles everything: 2 (above + diagonal / 2));
    // scaling the accumulators in the middle of the loop instead costs a copy of all of them through the vector registers
    auto store = [&](int stage, bool halve) {
        char* base = lds + stage * 2 * STILE;
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            const int id = tid + SNT * i, row = id >> 3, kc = id & 7;
            if (halve) {
                h8 x = __builtin_bit_cast(h8, ra[i]);
                x *= (_Float16)0.5f;
                ra[i] = __builtin_bit_cast(u4, x);
            }
            *reinterpret_cast<u4*>(base + row * SROW + kc * 16) = ra[i];
            *reinterpret_cast<u4*>(base + STILE + row * SROW + kc * 16) = rb[i];
        }
    };

    f16v acc[BLK][BLK];
#pragma unroll
    for (int a = 0; a < BLK; ++a)
#pragma unroll
        for (int b = 0; b < BLK; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    load(0);
    store(0, diag_step == 0);
    __syncthreads();
    for (int step = 0; step < n_steps; ++step) {
        if (step + 1 < n_steps) load(step + 1);                    // in flight behind this step's matrix work
        const char* At = lds + (step & 1) * 2 * STILE;
        const char* Bt = At + STILE;
        // v_mfma_f32_32x32x16_f16: lane l feeds row (column) l % 32 with the 8 contraction indices 8 (l / 32) .. + 8
        const int frow = lane & 31, fk = (lane >> 5) * 16;         // byte offset of the lane's 8 values inside a 16-wide group
#pragma unroll
        for (int kg = 0; kg < SK / 16; ++kg) {
            h8 af[BLK], bf[BLK];
#pragma unroll
            for (int a = 0; a < BLK; ++a) af[a] = *reinterpret_cast<const h8*>(At + (wr + 32 * a + frow) * SROW + kg * 32 + fk);
#pragma unroll
            for (int b = 0; b < BLK; ++b) bf[b] = *reinterpret_cast<const h8*>(Bt + (wc + 32 * b + frow) * SROW + kg * 32 + fk);
#pragma unroll
            for (int a = 0; a < BLK; ++a)
#pragma unroll
                for (int b = 0; b < BLK; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[a], bf[b], acc[a][b], 0, 0, 0);
        }
        if (step + 1 < n_steps) store((step + 1) & 1, step + 1 >= diag_step);      // the other stage: everybody left it before the last barrier
        __syncthreads();
    }

    // 32 x 32 result block: lane l, element v -> row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32
#pragma unroll
    for (int a = 0; a < BLK; ++a) {
        float s[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int64_t j = j0 + wr + 32 * a + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            float t = 0.0f;
#pragma unroll
            for (int b = 0; b < BLK; ++b) t = fmaf(acc[a][b][v], (float)E[j * d_in + c0 + wc + 32 * b + (lane & 31)], t);
            s[v] = t;
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {                             // over the 32 lanes that hold the row's columns, fixed order
            float t = s[v];
#pragma unroll
            for (int o = 16; o; o >>= 1) t += __shfl_xor(t, o);
            if ((lane & 31) == 0) {
                const int64_t j = j0 + wr + 32 * a + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                partial[((int64_t)cb * WPR + (wave % WPR)) * rows + j] = 2.0f * t;
            }
        }
    }
}

// ---- the same product on the pipelined 256 x 256 tile of tile256.h (d_in a multiple of 256)
//
// tile256 wants both operands contraction-major, so the residuals are kept transposed: Ft [d_in][rows] (row k holds f_k of
// every column of W).  The tile is C^T: its 256 rows are a column block cb of R (R is symmetric: row k of R, elements
// c0 .. c0+255), its 256 columns are columns j0 .. j0+255 of W; the contraction runs over k < 256 (cb + 1), and for the
// steps of the diagonal block the R rows come from Rh, a copy of R whose diagonal 256 x 256 blocks are halved (the
// epilogue doubles everything: 2 (above + diagonal / 2)).  A lane then holds one column j and 64 values of c per 32 x 32
// block, so the epilogue's sum over c of C[c][j] f_c[j] is a sum inside the lane plus one exchange between its two halves,
// and its reads of Ft are contiguous across the lanes.  partial[cb * 2 + h][j]: the sum over the 128 rows c of half h.

// Rh[c][k] = R[c][k] / 2 inside the diagonal 256 x 256 blocks, R[c][k] elsewhere
__global__ __launch_bounds__(256) void owc_corr_half_diag_kernel(const _Float16* __restrict__ R, int64_t d_in, _Float16* __restrict__ Rh) {
    const int64_t c = blockIdx.x;
    for (int64_t k = threadIdx.x; k < d_in; k += 256) {
        const _Float16 v = R[c * d_in + k];
        Rh[c * d_in + k] = (k / 256 == c / 256) ? (_Float16)(v * (_Float16)0.5f) : v;
    }
}

// largest d[k]
__global__ __launch_bounds__(1024) void owc_dmax_kernel(const float* __restrict__ d, int64_t d_in, float* __restrict__ out) {
    __shared__ float sh[16];
    float m = 0.0f;
    for (int64_t k = threadIdx.x; k < d_in; k += 1024) m = fmaxf(m, d[k]);
    for (int o = 32; o; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 16; ++w) m = fmaxf(m, sh[w]);
        out[0] = m;
    }
}

// Eq. (2) at one clipping strength for 64 columns of W and 1024 coordinates, stored transposed: Ft[k][j] = f_k / s_j in fp16,
// f = e * d with e = fma(a, q, lo) - w as the loss kernel forms it.  Here s_j is not the largest |f| of the column but a
// bound on it that needs no pass over the column: |e| <= max(a / 2, (hi - lo) - a (2^bits - 1)) -- half a step inside the
// grid, the clipped part above it -- times the largest d.  Any s that keeps |f / s| <= 1 serves (fp16 has the same
// relative precision over its whole normal range); s^2 goes to row_scale2.  Columns past d_out are written as zeros.
// 64 x 64 pieces go through LDS so that both the reads of W and the writes of Ft are contiguous.
__global__ __launch_bounds__(256) void owc_residual_f16_t_kernel(const float* __restrict__ Wt, int64_t d_out, int64_t d_in, int bits,
                                                                 const float* __restrict__ lo_in, const float* __restrict__ hi_in, float gamma,
                                                                 const float* __restrict__ d, const float* __restrict__ dmax,
                                                                 _Float16* __restrict__ Ft, int64_t rows, float* __restrict__ row_scale2) {
    constexpr int TS = 68;                                                   // halves per tile row: 136 bytes, 8-byte aligned
    __shared__ __attribute__((aligned(16))) _Float16 tile[64][TS];          // [j][k]
    __shared__ float a_sh[64], lo_sh[64], rs_sh[64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t j0 = (int64_t)blockIdx.x * 64, kb = (int64_t)blockIdx.y * 1024;
    const float top = (float)((1 << bits) - 1);
    if (tid < 64) {                                      // the columns' grids and scales
        const int64_t j = j0 + tid;
        float a = 1.0f, lo = 0.0f, rs = 0.0f;
        if (j < d_out) {
            lo = lo_in[j];
            const float hi = hi_in[j];
            a = __fdiv_rn(gamma * (hi - lo), top);
            if (!(a > 0.0f) || isinf(a)) a = 1.0f;
            float sc = fmaxf(0.5f * a, (hi - lo) - a * top) * dmax[0] * 1.001f;
            if (!(sc > 0.0f) || isinf(sc)) sc = 1.0f;
            rs = __fdiv_rn(1.0f, sc);
            if (blockIdx.y == 0) row_scale2[j] = sc * sc;
        }
        a_sh[tid] = a;
        lo_sh[tid] = lo;
        rs_sh[tid] = rs;                                 // 0 for a column past d_out: its entries become zeros
    }
    __syncthreads();
    // reading: per instruction a wavefront takes 4 columns x 64 coordinates (16 lanes x 4 consecutive floats each)
    const int rq = (lane & 15) * 4, rr = wave * 4 + (lane >> 4);
    // writing: coordinate wk, columns 16 wg .. 16 wg + 15
    const int wk = tid >> 2, wg = tid & 3;
    for (int64_t k0 = kb; k0 < kb + 1024 && k0 < d_in; k0 += 64) {
        const bool k_ok = k0 + rq < d_in;                // d_in is a multiple of 128 here, so a float4 is inside or outside
        const float4 dd = k_ok ? *reinterpret_cast<const float4*>(d + k0 + rq) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = i * 16 + rr;
            const float a = a_sh[row], lo = lo_sh[row], rs = rs_sh[row];
            float4 w = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (k_ok && rs != 0.0f) w = *reinterpret_cast<const float4*>(Wt + (j0 + row) * d_in + k0 + rq);
            auto f_one = [&](float wv, float dk) {
                const float q = fminf(fmaxf(rintf(__fdiv_rn(wv - lo, a)), 0.0f), top);
                return ((fmaf(a, q, lo) - wv) * dk) * rs;
            };
            typedef _Float16 h4 __attribute__((ext_vector_type(4)));
            h4 o;
            o.x = (_Float16)f_one(w.x, dd.x), o.y = (_Float16)f_one(w.y, dd.y), o.z = (_Float16)f_one(w.z, dd.z), o.w = (_Float16)f_one(w.w, dd.w);
            *reinterpret_cast<h4*>(&tile[row][rq]) = o;
        }
        __syncthreads();
        if (k0 + wk < d_in) {
            typedef _Float16 h8 __attribute__((ext_vector_type(8)));
            h8 o0, o1;
#pragma unroll
            for (int i = 0; i < 8; ++i) { o0[i] = tile[wg * 16 + i][wk]; o1[i] = tile[wg * 16 + 8 + i][wk]; }
            h8* dst = reinterpret_cast<h8*>(Ft + (k0 + wk) * rows + j0 + wg * 16);
            dst[0] = o0;
            dst[1] = o1;
        }
        __syncthreads();
    }
}

// grid.x = (d_in / 256) * (rows / 256) tiles, longest column blocks first.  Workgroup w runs on XCD w % 8 and each XCD has its
// own L2, so the tiles are handed out in patches of 4 column blocks of R x 8 blocks of columns of W, one patch per XCD at a
// time: its 32 tiles start at the same contraction index and read 12 operand blocks per step between them instead of 33.
// Shapes that do not divide into patches keep the plain order (same column block of R, consecutive columns of W).
__global__ __launch_bounds__(256) void owc_screen_t256_kernel(const _Float16* __restrict__ Ft, const _Float16* __restrict__ R,
                                                              const _Float16* __restrict__ Rh, int64_t rows, int64_t d_in,
                                                              float* __restrict__ partial) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int n_jt = (int)(rows / 256), n_cb = (int)(d_in / 256);
    int cb = n_cb - 1 - (int)(blockIdx.x / n_jt), jt = (int)(blockIdx.x % n_jt);
    if (n_cb % 4 == 0 && n_jt % 8 == 0 && ((n_cb / 4) * (n_jt / 8)) % 8 == 0) {
        const int xcd = (int)(blockIdx.x % 8), slot = (int)(blockIdx.x / 8);
        const int patch = (slot / 32) * 8 + xcd, t = slot % 32, n_jg = n_jt / 8;
        cb = n_cb - 1 - ((patch / n_jg) * 4 + t / 8);
        jt = (patch % n_jg) * 8 + t % 8;
    }
    const int64_t c0 = (int64_t)cb * 256, j0 = (int64_t)jt * 256;
    const int n_steps = (cb + 1) * (256 / tile256::BKS), alt_from = cb * (256 / tile256::BKS);
    tile256::acc16 acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;
    tile256::pipelined<tile256::F16>(reinterpret_cast<const char*>(R + c0), d_in * 2, reinterpret_cast<const char*>(Rh + c0), alt_from,
                                     reinterpret_cast<const char*>(Ft + j0), rows * 2, n_steps, lds, acc);
    // 32x32 block: lane l, element v -> row (c) 8*(v/4) + 4*(l/32) + v%4, column (j) l%32
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int64_t j = j0 + wn * 128 + b * 32 + (lane & 31);
        const _Float16* col = Ft + (c0 + wm * 128 + 4 * (lane >> 5)) * rows + j;
        float t = 0.0f;
        // the residuals of two 32-row blocks are fetched together, then used: left to itself the compiler waits for every
        // two-byte load before it issues the next, 256 round trips to L2 per tile
#pragma unroll
        for (int a2 = 0; a2 < 4; a2 += 2) {
            _Float16 f[2][16];
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int v = 0; v < 16; ++v) f[u][v] = col[(int64_t)((a2 + u) * 32 + 8 * (v >> 2) + (v & 3)) * rows];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int v = 0; v < 16; ++v) t = fmaf(acc[a2 + u][b][v], (float)f[u][v], t);
            __builtin_amdgcn_sched_barrier(0);
        }
        t += __shfl_xor(t, 32);
        if (lane < 32) partial[((int64_t)cb * 2 + wm) * rows + j] = 2.0f * t;
    }
}

// screened loss of a column at this grid point: the partial sums in a fixed order
__global__ __launch_bounds__(256) void owc_screen_rows_kernel(const float* __restrict__ partial, int64_t rows, int64_t d_out, int n_part,
                                                              const float* __restrict__ row_scale2, float* __restrict__ out) {
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= d_out) return;
    float s = 0.0f;
    for (int p = 0; p < n_part; ++p) s += partial[(int64_t)p * rows + j];
    out[j] = s * row_scale2[j];
}

// Per column: the grid points whose screened loss is within the margin of the smallest, best first.  cand [n_gamma][d_out]:
// grid index k (1-based) of the column's r-th candidate, 0 when it has fewer; active [n_gamma][row blocks of the loss kernel]:
// set when some column of the block has an r-th candidate (zeroed by the caller).  A NaN counts as a candidate.
__global__ __launch_bounds__(256) void owc_rank_kernel(const float* __restrict__ screened, int64_t d_out, int n_gamma, float margin,
                                                       int block_rows, int64_t n_blocks, uint8_t* __restrict__ cand,
                                                       uint8_t* __restrict__ active) {
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= d_out) return;
    float best = INFINITY;
    for (int k = 0; k < n_gamma; ++k) {
        const float v = screened[(int64_t)k * d_out + j];
        if (v < best) best = v;
    }
    const float limit = best + margin * fabsf(best) + 1e-30f;
    // selection by repeated minimum over what is left: n_gamma is small
    float prev = -INFINITY;
    int prev_k = -1, r = 0;
    for (;; ++r) {
        float cur = INFINITY;
        int cur_k = -1;
        for (int k = 0; k < n_gamma; ++k) {
            float v = screened[(int64_t)k * d_out + j];
            if (!(v == v)) v = -INFINITY;                          // a NaN sorts first: it is evaluated exactly
            if (!(v <= limit)) continue;
            if ((v > prev || (v == prev && k > prev_k)) && (cur_k < 0 || v < cur)) { cur = v; cur_k = k; }
        }
        if (cur_k < 0) break;
        cand[(int64_t)r * d_out + j] = (uint8_t)(cur_k + 1);
        active[(int64_t)r * n_blocks + j / block_rows] = 1;
        prev = cur;
        prev_k = cur_k;
    }
    for (; r < n_gamma; ++r) cand[(int64_t)r * d_out + j] = 0;
}

}  // namespace

bool owc_screen_applies(int64_t d_out, int64_t d_in, int n_gamma) {
    return d_in % SB == 0 && d_in >= 2 * SB && n_gamma >= 4 && n_gamma <= 255 && d_out >= 1 && d_in / SB * 2 <= 0x7fffffffLL;
}

// R [d_in][d_in] fp16 | Rh (R with halved diagonal blocks) | F [rows][d_in] fp16 (Ft [d_in][rows] on the 256-wide path) | partial [2 d_in / SB][rows] fp32 | screened [n_gamma][d_out] fp32 |
// cand [n_gamma][d_out] u8 | active [n_gamma][n_blocks] u8 | d, 1/d [d_in] fp32 each | row scales [d_out] fp32
size_t owc_screen_workspace_bytes(int64_t d_out, int64_t d_in, int n_gamma, int64_t n_blocks) {
    const int64_t rows = (d_out + 2 * SB - 1) / (2 * SB) * (2 * SB);
    return 2 * cdq_align_up((size_t)d_in * d_in * 2, 256) + cdq_align_up((size_t)rows * d_in * 2, 256) +
           cdq_align_up((size_t)(2 * d_in / SB) * rows * sizeof(float), 256) + cdq_align_up((size_t)n_gamma * d_out * sizeof(float), 256) +
           cdq_align_up((size_t)n_gamma * d_out, 256) + cdq_align_up((size_t)n_gamma * n_blocks, 256) +
           2 * cdq_align_up((size_t)d_in * sizeof(float), 256) + cdq_align_up((size_t)d_out * sizeof(float), 256) + 256;
}

// Screens all n_gamma grid points and ranks them.  On return (stream order) cand, active and the screened losses
// [n_gamma][d_out] are filled; all three point into ws.
int owc_screen_launch(const float* H, const float* Wt, int64_t d_out, int64_t d_in, int bits, int n_gamma, const float* lo, const float* hi,
                      float margin, int block_rows, int64_t n_blocks, void* ws, uint8_t** cand_out, uint8_t** active_out,
                      const float** screened_out, hipStream_t st) {
    const int64_t rows = (d_out + 2 * SB - 1) / (2 * SB) * (2 * SB);
    const int n_part = (int)(2 * d_in / SB);
    const bool big = d_in % (2 * SB) == 0;                         // the 256 x 256 tile
    const int n_sum = n_part;                                      // partial sums per row that the kernel writes
    char* p = (char*)ws;
    _Float16* R = (_Float16*)p;        p += cdq_align_up((size_t)d_in * d_in * 2, 256);
    _Float16* Rh = (_Float16*)p;       p += cdq_align_up((size_t)d_in * d_in * 2, 256);
    _Float16* F = (_Float16*)p;        p += cdq_align_up((size_t)rows * d_in * 2, 256);
    float* partial = (float*)p;        p += cdq_align_up((size_t)n_part * rows * sizeof(float), 256);
    float* screened = (float*)p;       p += cdq_align_up((size_t)n_gamma * d_out * sizeof(float), 256);
    uint8_t* cand = (uint8_t*)p;       p += cdq_align_up((size_t)n_gamma * d_out, 256);
    uint8_t* active = (uint8_t*)p;     p += cdq_align_up((size_t)n_gamma * n_blocks, 256);
    float* d = (float*)p;              p += cdq_align_up((size_t)d_in * sizeof(float), 256);
    float* rd = (float*)p;             p += cdq_align_up((size_t)d_in * sizeof(float), 256);
    float* row_scale2 = (float*)p;     p += cdq_align_up((size_t)d_out * sizeof(float), 256);
    float* dmax = (float*)p;
    if (rows / SB > 65535) return CDQ_EUNSUPPORTED;
    hipLaunchKernelGGL(owc_diag_kernel, dim3((unsigned)((d_in + 255) / 256)), dim3(256), 0, st, H, d_in, d, rd);
    CDQ_LAUNCH_CHECK();
    hipLaunchKernelGGL(owc_corr_f16_kernel, dim3((unsigned)d_in), dim3(256), 0, st, H, d_in, (const float*)rd, R);
    CDQ_LAUNCH_CHECK();
    const bool t256 = big && d_in <= 65536 && rows * 2 <= 128 * 1024;      // the pipelined tile: rows of Ft at most 128 KiB apart
    if (t256) {
        hipLaunchKernelGGL(owc_corr_half_diag_kernel, dim3((unsigned)d_in), dim3(256), 0, st, (const _Float16*)R, d_in, Rh);
        CDQ_LAUNCH_CHECK();
        hipLaunchKernelGGL(owc_dmax_kernel, dim3(1), dim3(1024), 0, st, (const float*)d, d_in, dmax);
        CDQ_LAUNCH_CHECK();
    }
    if (rows > d_out && !t256) {                                   // d_in is a multiple of 128: whole words
        const int64_t words = (rows - d_out) * d_in / 2;
        hipLaunchKernelGGL(fill_words_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st, (uint32_t*)(F + d_out * d_in), words, 0u);
        CDQ_LAUNCH_CHECK();
    }
    {
        const int64_t words = (int64_t)(cdq_align_up((size_t)n_gamma * n_blocks, 256) / 4);     // the region is padded to 256 bytes
        hipLaunchKernelGGL(fill_words_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st, (uint32_t*)active, words, 0u);
        CDQ_LAUNCH_CHECK();
    }
    constexpr int lds_small = 2 * 2 * SB * SROW, lds_big = 2 * 2 * 2 * SB * SROW;
    static const hipError_t lds_rc_small = hipFuncSetAttribute(reinterpret_cast<const void*>(owc_screen_kernel<SB, 2>),
                                                               hipFuncAttributeMaxDynamicSharedMemorySize, lds_small);
    static const hipError_t lds_rc_big = hipFuncSetAttribute(reinterpret_cast<const void*>(owc_screen_kernel<2 * SB, 2>),
                                                             hipFuncAttributeMaxDynamicSharedMemorySize, lds_big);
    static const hipError_t lds_rc_t256 = hipFuncSetAttribute(reinterpret_cast<const void*>(owc_screen_t256_kernel),
                                                              hipFuncAttributeMaxDynamicSharedMemorySize, tile256::LDS_BYTES);
    if (lds_rc_small != hipSuccess || lds_rc_big != hipSuccess || lds_rc_t256 != hipSuccess) return CDQ_EHIP;
    for (int k = 1; k <= n_gamma; ++k) {
        const float gamma = (float)k / (float)n_gamma;
        if (t256) {
            hipLaunchKernelGGL(owc_residual_f16_t_kernel, dim3((unsigned)(rows / 64), (unsigned)((d_in + 1023) / 1024)), dim3(256), 0, st, Wt, d_out,
                               d_in, bits, lo, hi, gamma, (const float*)d, (const float*)dmax, F, rows, row_scale2);
            CDQ_LAUNCH_CHECK();
            hipLaunchKernelGGL(owc_screen_t256_kernel, dim3((unsigned)((d_in / 256) * (rows / 256))), dim3(256), tile256::LDS_BYTES, st,
                               (const _Float16*)F, (const _Float16*)R, (const _Float16*)Rh, rows, d_in, partial);
            CDQ_LAUNCH_CHECK();
            hipLaunchKernelGGL(owc_screen_rows_kernel, dim3((unsigned)((d_out + 255) / 256)), dim3(256), 0, st, (const float*)partial, rows,
                               d_out, (int)(d_in / 128), (const float*)row_scale2, screened + (int64_t)(k - 1) * d_out);
            CDQ_LAUNCH_CHECK();
            continue;
        }
        if (((uintptr_t)Wt & 15) == 0)
            hipLaunchKernelGGL(owc_residual_f16_vec_kernel, dim3((unsigned)d_out), dim3(256), 0, st, Wt, d_in, bits, lo, hi, gamma,
                               (const float*)d, F, row_scale2);
        else
            hipLaunchKernelGGL(owc_residual_f16_kernel, dim3((unsigned)d_out), dim3(256), 0, st, Wt, d_in, bits, lo, hi, gamma,
                               (const float*)d, F, row_scale2);
        CDQ_LAUNCH_CHECK();
        if (big)
            hipLaunchKernelGGL((owc_screen_kernel<2 * SB, 2>), dim3((unsigned)(d_in / (2 * SB)), (unsigned)(rows / (2 * SB))), dim3(1024), lds_big, st,
                               (const _Float16*)F, (const _Float16*)R, rows, d_in, partial);
        else
            hipLaunchKernelGGL((owc_screen_kernel<SB, 2>), dim3((unsigned)(d_in / SB), (unsigned)(rows / SB)), dim3(256), lds_small, st,
                               (const _Float16*)F, (const _Float16*)R, rows, d_in, partial);
        CDQ_LAUNCH_CHECK();
        hipLaunchKernelGGL(owc_screen_rows_kernel, dim3((unsigned)((d_out + 255) / 256)), dim3(256), 0, st, (const float*)partial, rows,
                           d_out, n_sum, (const float*)row_scale2, screened + (int64_t)(k - 1) * d_out);
        CDQ_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(owc_rank_kernel, dim3((unsigned)((d_out + 255) / 256)), dim3(256), 0, st, (const float*)screened, d_out, n_gamma,
                       margin, block_rows, n_blocks, cand, active);
    CDQ_LAUNCH_CHECK();
    *cand_out = cand;
    *active_out = active;
    *screened_out = screened;
    return CDQ_OK;
}

}  // namespace cdq
