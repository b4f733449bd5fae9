// Optimal Weight Clipping (paper Section 3.1, "Initializing a, b, q"; Eq. (2)): per output column,
// grid search over the clipping strength gamma for the smallest layer loss of Eq. (1).
//   b = min w,  a(gamma) = gamma (max w - min w)/(2^c - 1),  q = clamp(round((w - b)/a), 0, 2^c - 1)
// The grid is gamma_k = k/n_gamma, k = 1..n_gamma (gamma = 1 is MinMax; equal losses keep the
// larger gamma).  A grid point costs one pass of the fp64 loss kernel over all columns; where the fp16 look at all grid
// points applies (owc_screen.hip) only the few that can win are evaluated that way: every column's best-screened point in
// one pass over all columns, the check of the look against that value, the other candidates gathered into dense rows, and
// what does not fit the rows one rank at a time, blocks of columns without a candidate of that rank skipped.
#include "cdq_internal.h"

namespace cdq {
namespace {

__device__ __forceinline__ float wave_min(float v) { for (int o = 32; o; o >>= 1) v = fminf(v, __shfl_xor(v, o)); return v; }
__device__ __forceinline__ float wave_max(float v) { for (int o = 32; o; o >>= 1) v = fmaxf(v, __shfl_xor(v, o)); return v; }

// one workgroup per column: lo = min w, hi = max w
__global__ __launch_bounds__(256) void owc_minmax_kernel(const float* __restrict__ Wt, int64_t d_in, float* __restrict__ lo_out,
                                                         float* __restrict__ hi_out) {
    __shared__ float slo[4], shi[4];
    const int64_t j = blockIdx.x;
    const float* w = Wt + j * d_in;
    float lo = INFINITY, hi = -INFINITY;
    for (int64_t k = threadIdx.x; k < d_in; k += 256) {
        const float v = w[k];
        lo = fminf(lo, v);
        hi = fmaxf(hi, v);
    }
    lo = wave_min(lo);
    hi = wave_max(hi);
    if ((threadIdx.x & 63) == 0) { slo[threadIdx.x >> 6] = lo; shi[threadIdx.x >> 6] = hi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        lo_out[j] = fminf(fminf(slo[0], slo[1]), fminf(slo[2], slo[3]));
        hi_out[j] = fmaxf(fmaxf(shi[0], shi[1]), fmaxf(shi[2], shi[3]));
    }
}

// Eq. (2) for one clipping strength: uniform gamma (gamma_col == nullptr) or one per column
__global__ __launch_bounds__(256) void owc_quantize_kernel(const float* __restrict__ Wt, int64_t d_in, int bits,
                                                           const float* __restrict__ lo_in, const float* __restrict__ hi_in,
                                                           float gamma, const float* __restrict__ gamma_col,
                                                           float* __restrict__ scale, float* __restrict__ zero,
                                                           uint8_t* __restrict__ Q) {
    const int64_t j = blockIdx.x;
    const float lo = lo_in[j], hi = hi_in[j];
    const float g = gamma_col ? gamma_col[j] : gamma;
    if (!(g > 0.0f)) return;                                              // no grid point for this column in this pass
    const float top = (float)((1 << bits) - 1);
    float a = __fdiv_rn(g * (hi - lo), top);
    if (!(a > 0.0f) || isinf(a)) a = 1.0f;
    if (threadIdx.x == 0) {
        scale[j] = a;
        if (zero != nullptr) zero[j] = lo;
    }
    const float* w = Wt + j * d_in;
    uint8_t* q = Q + j * d_in;
    for (int64_t k = threadIdx.x; k < d_in; k += 256) {
        const float t = __fdiv_rn(w[k] - lo, a);
        q[k] = (uint8_t)fminf(fmaxf(rintf(t), 0.0f), top);
    }
}

__global__ __launch_bounds__(256) void owc_update_best_kernel(const double* __restrict__ cur, int64_t d_out, float gamma, int first,
                                                              double* __restrict__ best, float* __restrict__ best_gamma) {
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= d_out) return;
    const double c = cur[j];
    if (first || c <= best[j]) {          // "<=": equal losses keep the larger gamma (gammas ascend)
        best[j] = c;
        best_gamma[j] = gamma;
    }
}

// rank r of the candidates: the column's gamma (0: none) for the quantize pass
__global__ __launch_bounds__(256) void owc_rank_gamma_kernel(const uint8_t* __restrict__ cand_r, int64_t d_out, int n_gamma,
                                                             float* __restrict__ gamma_col) {
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= d_out) return;
    const int k = cand_r[j];
    gamma_col[j] = k ? (float)k / (float)n_gamma : 0.0f;
}

// exact losses of one rank folded into the best: smaller wins, equal losses keep the larger gamma -- the result of going
// through the grid in ascending order with "<=", whatever the order of the ranks
__global__ __launch_bounds__(256) void owc_update_best_ranked_kernel(const double* __restrict__ cur, const float* __restrict__ gamma_col,
                                                                     int64_t d_out, double* __restrict__ best,
                                                                     float* __restrict__ best_gamma) {
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= d_out) return;
    const float g = gamma_col[j];
    if (!(g > 0.0f)) return;
    const double c = cur[j];
    const float bg = best_gamma[j];
    if (bg == 0.0f || c < best[j] || (c == best[j] && g > bg)) {
        best[j] = c;
        best_gamma[j] = g;
    }
}

__global__ __launch_bounds__(256) void owc_fill_u8_kernel(uint8_t* __restrict__ p, int64_t n, uint8_t v) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}

__global__ __launch_bounds__(256) void owc_fill_f32_kernel(float* __restrict__ p, int64_t n, float v) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}

// ---- candidates gathered into dense rows for one pass of the loss kernel.  first = 1: every column's best-screened
// candidate is evaluated with all columns in a pass of its own (the caller wants each column's loss) and the rows take the
// others; first = 0: a column with a single candidate needs no evaluation at all, and the rows take all candidates of the
// columns that have several.
// extras[j]: how many rows column j asks for (cand [n_gamma][d_out], a column's candidates are contiguous in r)
__global__ __launch_bounds__(256) void owc_count_extras_kernel(const uint8_t* __restrict__ cand, int64_t d_out, int n_gamma, int first,
                                                               int32_t* __restrict__ extras) {
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= d_out) return;
    int n = 0;
    for (int r = 0; r < n_gamma && cand[(int64_t)r * d_out + j] != 0; ++r) ++n;
    extras[j] = first == 1 ? (n > 0 ? n - 1 : 0) : (n >= 2 ? n : 0);
}

// base[j] = extras[0] + ... + extras[j-1]; one workgroup, the columns in chunks of 1024; total is cleared
__global__ __launch_bounds__(1024) void owc_scan_extras_kernel(const int32_t* __restrict__ extras, int64_t d_out, int32_t* __restrict__ base,
                                                               int32_t* __restrict__ total) {
    __shared__ int32_t sh[1024];
    __shared__ int32_t carry;
    if (threadIdx.x == 0) { carry = 0; *total = 0; }
    __syncthreads();
    for (int64_t j0 = 0; j0 < d_out; j0 += 1024) {
        const int64_t j = j0 + threadIdx.x;
        const int32_t v = j < d_out ? extras[j] : 0;
        sh[threadIdx.x] = v;
        __syncthreads();
        for (int o = 1; o < 1024; o <<= 1) {                       // inclusive scan of the chunk
            const int32_t t = (int)threadIdx.x >= o ? sh[threadIdx.x - o] : 0;
            __syncthreads();
            sh[threadIdx.x] += t;
            __syncthreads();
        }
        if (j < d_out) base[j] = carry + sh[threadIdx.x] - v;
        __syncthreads();
        if (threadIdx.x == 1023) carry += sh[1023];
        __syncthreads();
    }
}

// A column whose rows fit below cap gets rows base[j] .. base[j] + extras[j] - 1 for its candidates first, first + 1, ...:
// their column and grid index are recorded, they are struck from cand (the rank passes will not see them), total becomes
// the number of rows in use.  With first = 0 a column with one candidate takes that grid point without evaluation.
__global__ __launch_bounds__(256) void owc_assign_rows_kernel(uint8_t* __restrict__ cand, int64_t d_out, int n_gamma, int first,
                                                              const int32_t* __restrict__ extras, const int32_t* __restrict__ base,
                                                              int32_t cap, int32_t* __restrict__ row_col, uint8_t* __restrict__ row_k,
                                                              int32_t* __restrict__ total, float* __restrict__ best_gamma) {
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= d_out) return;
    const int32_t e = extras[j], b = base[j];
    if (first == 0 && e == 0 && cand[j] != 0 && (n_gamma < 2 || cand[d_out + j] == 0)) {
        best_gamma[j] = (float)cand[j] / (float)n_gamma;
        cand[j] = 0;
        return;
    }
    if (e == 0 || (int64_t)b + e > cap) return;
    for (int r = 0; r < e; ++r) {
        row_col[b + r] = (int32_t)j;
        row_k[b + r] = cand[(int64_t)(first + r) * d_out + j];
        cand[(int64_t)(first + r) * d_out + j] = 0;
    }
    atomicMax(total, b + e);
}

// which blocks of the loss kernel have work: rank r >= first of the columns (what the rows above did not take; the flags of
// those ranks were cleared by the caller), and the rows
__global__ __launch_bounds__(256) void owc_flags_kernel(const uint8_t* __restrict__ cand, int64_t d_out, int n_gamma, int first, int block_rows,
                                                        int64_t n_blocks, const int32_t* __restrict__ total, uint8_t* __restrict__ active,
                                                        uint8_t* __restrict__ rows_active) {
    const int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x;     // over (r, j), r >= first
    if (x < n_blocks) rows_active[x] = (x * block_rows < *total) ? 1 : 0;
    if (x >= (int64_t)(n_gamma - first) * d_out) return;
    const int64_t r = first + x / d_out, j = x % d_out;
    if (cand[r * d_out + j] != 0) active[r * n_blocks + j / block_rows] = 1;
}

// row s < total: minus the residual of its column at its grid point, so that the loss kernel, given scale = zero = 0,
// forms e = fma(0, q, 0) - (w - fma(a, q, lo)) -- the same bits as fma(a, q, lo) - w
__global__ __launch_bounds__(256) void owc_row_residual_kernel(const float* __restrict__ Wt, int64_t d_in, int bits, const float* __restrict__ lo_in,
                                                               const float* __restrict__ hi_in, int n_gamma, const int32_t* __restrict__ row_col,
                                                               const uint8_t* __restrict__ row_k, const int32_t* __restrict__ total,
                                                               float* __restrict__ Wc) {
    const int64_t s = blockIdx.x;
    if (s >= *total) return;
    const int64_t j = row_col[s];
    const float lo = lo_in[j], hi = hi_in[j];
    const float g = (float)row_k[s] / (float)n_gamma;
    const float top = (float)((1 << bits) - 1);
    float a = __fdiv_rn(g * (hi - lo), top);
    if (!(a > 0.0f) || isinf(a)) a = 1.0f;
    const float* w = Wt + j * d_in;
    float* o = Wc + s * d_in;
    for (int64_t k = threadIdx.x; k < d_in; k += 256) {
        const float wk = w[k];
        const float q = fminf(fmaxf(rintf(__fdiv_rn(wk - lo, a)), 0.0f), top);
        o[k] = wk - fmaf(a, q, lo);
    }
}

__global__ __launch_bounds__(256) void owc_update_best_rows_kernel(const double* __restrict__ row_loss, const uint8_t* __restrict__ row_k,
                                                                   const int32_t* __restrict__ extras, const int32_t* __restrict__ base,
                                                                   int32_t cap, int n_gamma, int64_t d_out, double* __restrict__ best,
                                                                   float* __restrict__ best_gamma) {
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= d_out) return;
    const int32_t e = extras[j], b = base[j];
    if (e == 0 || (int64_t)b + e > cap) return;
    double bl = best[j];
    float bg = best_gamma[j];
    for (int r = 0; r < e; ++r) {
        const double c = row_loss[b + r];
        const float g = (float)row_k[b + r] / (float)n_gamma;
        if (bg == 0.0f || c < bl || (c == bl && g > bg)) { bl = c; bg = g; }
    }
    best[j] = bl;
    best_gamma[j] = bg;
}

// ---- the start gradient as a by-product: the pass over every column's best-screened grid point leaves H e of that grid
// point in G; the columns that ended at another grid point get their row again.
// changed[j] = 1 where the chosen strength is not the one the row of G was computed for
__global__ __launch_bounds__(256) void owc_changed_kernel(const float* __restrict__ best_gamma, const float* __restrict__ first_gamma,
                                                          int64_t d_out, int32_t* __restrict__ changed) {
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j < d_out) changed[j] = best_gamma[j] != first_gamma[j] ? 1 : 0;
}

// the changed columns, in order, as rows: row base[j] is column j at its chosen grid index; total = their number; flags for
// the blocks of rows that exist
__global__ __launch_bounds__(256) void owc_changed_rows_kernel(const int32_t* __restrict__ changed, const int32_t* __restrict__ base,
                                                               const float* __restrict__ best_gamma, int n_gamma, int64_t d_out,
                                                               int32_t* __restrict__ row_col, uint8_t* __restrict__ row_k,
                                                               int32_t* __restrict__ total) {
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= d_out || changed[j] == 0) return;
    int k = (int)rintf(best_gamma[j] * (float)n_gamma);
    k = k < 1 ? 1 : (k > n_gamma ? n_gamma : k);
    row_col[base[j]] = (int32_t)j;
    row_k[base[j]] = (uint8_t)k;
    atomicMax(total, base[j] + 1);
}

__global__ __launch_bounds__(256) void owc_row_blocks_kernel(const int32_t* __restrict__ total, int block_rows, int64_t n_blocks,
                                                             uint8_t* __restrict__ rows_active) {
    const int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (x < n_blocks) rows_active[x] = (x * block_rows < *total) ? 1 : 0;
}

constexpr float kScreenMargin = 3e-3f;      // relative; the fp16 evaluation was off by 3e-4 at most on heavy-tailed test layers

// The check that makes the two-stage search safe to use: every column's best-screened grid point has been evaluated both
// ways, so the error of the fp16 look on this column is known there.  Where it exceeds a third of the margin (or is not a
// number) the look is not trusted for the column: every other grid point becomes a candidate behind the one already
// evaluated (ranks 1 .. n_gamma - 1, ascending), to be evaluated in fp64 by the rows and rank passes that follow, and the
// column is counted.
__global__ __launch_bounds__(256) void owc_guard_kernel(const float* __restrict__ screened, const double* __restrict__ best_loss,
                                                        const float* __restrict__ best_gamma, int64_t d_out, int n_gamma, float margin,
                                                        uint8_t* __restrict__ cand, int32_t* __restrict__ count) {
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= d_out) return;
    const float g = best_gamma[j];
    int k = (int)rintf(g * (float)n_gamma);                    // best_gamma is k / n_gamma in fp32
    if (k < 1) k = 1;
    if (k > n_gamma) k = n_gamma;
    const double exact = best_loss[j], seen = (double)screened[(int64_t)(k - 1) * d_out + j];
    // a residual of zero (exact == 0: a constant column) is screened as zero too
    const bool trusted = (g > 0.0f) && (exact == seen || fabs(exact - seen) <= (double)(margin / 3.0f) * fabs(exact));
    if (trusted) return;
    cand[j] = (uint8_t)k;                                      // rank 0 stays what was evaluated
    int r = 1;
    for (int kk = 1; kk <= n_gamma; ++kk)
        if (kk != k) cand[(int64_t)(r++) * d_out + j] = (uint8_t)kk;
    atomicAdd(count, 1);
}

}  // namespace

size_t owc_workspace_bytes(int64_t d_out, int64_t d_in) {
    size_t b = 0;
    b += cdq_align_up((size_t)d_out * sizeof(float), 256) * 5;       // lo, hi, trial scale, best gamma, a rank's gammas
    b += cdq_align_up((size_t)d_out * sizeof(double), 256) * 2;      // trial loss, best loss
    b += cdq_align_up((size_t)d_out * d_in, 256);                    // trial codes
    b += loss_workspace_bytes(d_out, d_in);
    const int64_t n_blocks = (d_out + loss_block_rows() - 1) / loss_block_rows();
    b += owc_screen_workspace_bytes(d_out, d_in, 255, n_blocks);     // sized for the largest grid the screen takes
    // the gathered candidates: rows of minus-residuals [d_out][d_in], their losses, zeros for scale and zero, extras, base,
    // row -> column, row -> grid index, total, block flags
    b += cdq_align_up((size_t)d_out * d_in * sizeof(float), 256) + cdq_align_up((size_t)d_out * sizeof(double), 256);
    b += cdq_align_up((size_t)d_out * sizeof(float), 256) * 4 + cdq_align_up((size_t)d_out, 256) + 256 + cdq_align_up((size_t)n_blocks, 256);
    b += cdq_align_up((size_t)d_out * sizeof(float), 256);           // the strength each row of the start gradient was computed for
    return b;
}

int owc_launch(const float* H, const float* Wt, int64_t d_out, int64_t d_in, int bits, int n_gamma, float screen_margin, float* scale,
               float* zero, uint8_t* Q, float* gamma_out, double* loss_out, int32_t* researched, float* G_out, void* ws, size_t ws_bytes,
               hipStream_t st) {
    if (d_out == 0) {
        if (researched != nullptr) {
            hipLaunchKernelGGL(owc_fill_f32_kernel, dim3(1), dim3(256), 0, st, (float*)researched, (int64_t)1, 0.0f);     // the bits of +0.0f are the integer 0
            CDQ_LAUNCH_CHECK();
        }
        return CDQ_OK;
    }
    const float margin = screen_margin > 0.0f ? screen_margin : kScreenMargin;
    if (ws == nullptr || ((uintptr_t)ws & 255) || ws_bytes < owc_workspace_bytes(d_out, d_in)) return CDQ_EWORKSPACE;
    if (d_out > 0x7fffffffLL) return CDQ_EUNSUPPORTED;
    char* p = (char*)ws;
    const size_t fsz = cdq_align_up((size_t)d_out * sizeof(float), 256), dsz = cdq_align_up((size_t)d_out * sizeof(double), 256);
    float* lo = (float*)p; p += fsz;
    float* hi = (float*)p; p += fsz;
    float* trial_scale = (float*)p; p += fsz;
    float* best_gamma = (float*)p; p += fsz;
    float* rank_gamma = (float*)p; p += fsz;
    double* trial_loss = (double*)p; p += dsz;
    double* best_loss = (double*)p; p += dsz;
    uint8_t* trial_q = (uint8_t*)p; p += cdq_align_up((size_t)d_out * d_in, 256);
    void* loss_ws = p;
    const size_t loss_ws_bytes = loss_workspace_bytes(d_out, d_in);
    const dim3 cols((unsigned)d_out), t256(256);

    void* screen_ws = (char*)loss_ws + loss_ws_bytes;
    const dim3 col_blocks((unsigned)((d_out + 255) / 256));

    hipLaunchKernelGGL(owc_minmax_kernel, cols, t256, 0, st, Wt, d_in, lo, hi);
    CDQ_LAUNCH_CHECK();
    bool g_from_first_pass = false;
    float* first_gamma = nullptr;
    int32_t *g_changed = nullptr, *g_base = nullptr, *g_row_col = nullptr, *g_total = nullptr;
    uint8_t *g_row_k = nullptr, *g_rows_active = nullptr;
    float *g_Wc = nullptr, *g_zeros = nullptr;
    if (owc_screen_applies(d_out, d_in, n_gamma)) {
        const int block_rows = loss_block_rows();
        const int64_t n_blocks = (d_out + block_rows - 1) / block_rows;
        uint8_t *cand, *active;
        const float* screened;
        int rc = owc_screen_launch(H, Wt, d_out, d_in, bits, n_gamma, lo, hi, margin, block_rows, n_blocks, screen_ws, &cand, &active, &screened, st);
        if (rc != CDQ_OK) return rc;
        hipLaunchKernelGGL(owc_fill_f32_kernel, col_blocks, t256, 0, st, best_gamma, d_out, 0.0f);      // 0: nothing evaluated yet
        CDQ_LAUNCH_CHECK();
        // Every column's best-screened grid point is evaluated in fp64 in a pass over all columns (that value is also what the
        // check of the fp16 look compares with); the other candidates are gathered into at most d_out dense rows.
        const int first = 1;
        char* gp = (char*)screen_ws + owc_screen_workspace_bytes(d_out, d_in, 255, n_blocks);
        float* Wc = (float*)gp;             gp += cdq_align_up((size_t)d_out * d_in * sizeof(float), 256);
        double* row_loss = (double*)gp;     gp += dsz;
        float* zeros = (float*)gp;          gp += fsz;
        int32_t* extras = (int32_t*)gp;     gp += fsz;
        int32_t* base = (int32_t*)gp;       gp += fsz;
        int32_t* row_col = (int32_t*)gp;    gp += fsz;
        uint8_t* row_k = (uint8_t*)gp;      gp += cdq_align_up((size_t)d_out, 256);
        int32_t* total = (int32_t*)gp;      gp += 256;
        uint8_t* rows_active = (uint8_t*)gp;  gp += cdq_align_up((size_t)n_blocks, 256);
        first_gamma = (float*)gp;
        g_changed = extras; g_base = base; g_row_col = row_col; g_total = total; g_row_k = row_k; g_rows_active = rows_active;
        g_Wc = Wc; g_zeros = zeros;
        const int32_t cap = (int32_t)d_out;
        int32_t* count = total + 1;         // columns that fail the check (the scan clears total only)
        hipLaunchKernelGGL(owc_fill_f32_kernel, col_blocks, t256, 0, st, zeros, d_out, 0.0f);
        CDQ_LAUNCH_CHECK();
        hipLaunchKernelGGL(owc_fill_f32_kernel, dim3(1), t256, 0, st, (float*)count, (int64_t)1, 0.0f);                   // bits of +0.0f: integer 0
        CDQ_LAUNCH_CHECK();
        // rank passes: every column at its r-th candidate, blocks of columns without one skipped
        auto rank_pass = [&](int r) -> int {
            hipLaunchKernelGGL(owc_rank_gamma_kernel, col_blocks, t256, 0, st, cand + (int64_t)r * d_out, d_out, n_gamma, rank_gamma);
            CDQ_LAUNCH_CHECK();
            hipLaunchKernelGGL(owc_quantize_kernel, cols, t256, 0, st, Wt, d_in, bits, lo, hi, 1.0f, (const float*)rank_gamma, trial_scale,
                               (float*)nullptr, trial_q);
            CDQ_LAUNCH_CHECK();
            if (r == 0 && G_out != nullptr) {
                // every column is in this pass: the whole product, which leaves H e in G_out, with the loss taken from the same sums
                const int rc2 = gradient_loss_launch(H, Wt, trial_scale, lo, trial_q, d_out, d_in, d_in, G_out, trial_loss, loss_ws, loss_ws_bytes,
                                                     st, nullptr, nullptr, nullptr);
                if (rc2 != CDQ_OK) return rc2;
                CDQ_HIP_CHECK(hipMemcpyAsync(first_gamma, rank_gamma, (size_t)d_out * sizeof(float), hipMemcpyDeviceToDevice, st));
                g_from_first_pass = true;
            } else {
                const int rc2 = loss_launch(H, Wt, trial_scale, lo, trial_q, d_out, d_in, d_in, trial_loss, nullptr, loss_ws, loss_ws_bytes, st,
                                            active + (int64_t)r * n_blocks);
                if (rc2 != CDQ_OK) return rc2;
            }
            hipLaunchKernelGGL(owc_update_best_ranked_kernel, col_blocks, t256, 0, st, (const double*)trial_loss, (const float*)rank_gamma,
                               d_out, best_loss, best_gamma);
            CDQ_LAUNCH_CHECK();
            return CDQ_OK;
        };
        // 1. every column's best-screened grid point, in fp64
        rc = rank_pass(0);
        if (rc != CDQ_OK) return rc;
        // 2. the check of the fp16 look: a column that fails it gets every other grid point as a candidate
        hipLaunchKernelGGL(owc_guard_kernel, col_blocks, t256, 0, st, screened, (const double*)best_loss, (const float*)best_gamma, d_out, n_gamma,
                           margin, cand, count);
        CDQ_LAUNCH_CHECK();
        // 3. the candidates beyond the first, gathered into dense rows for one pass of the loss kernel ...
        hipLaunchKernelGGL(owc_count_extras_kernel, col_blocks, t256, 0, st, cand, d_out, n_gamma, first, extras);
        CDQ_LAUNCH_CHECK();
        hipLaunchKernelGGL(owc_scan_extras_kernel, dim3(1), dim3(1024), 0, st, (const int32_t*)extras, d_out, base, total);
        CDQ_LAUNCH_CHECK();
        hipLaunchKernelGGL(owc_assign_rows_kernel, col_blocks, t256, 0, st, cand, d_out, n_gamma, first, (const int32_t*)extras,
                           (const int32_t*)base, cap, row_col, row_k, total, best_gamma);
        CDQ_LAUNCH_CHECK();
        {
            const int64_t flags = (int64_t)(n_gamma - first) * n_blocks;             // ranks >= first start with no block active
            hipLaunchKernelGGL(owc_fill_u8_kernel, dim3((unsigned)((flags + 255) / 256)), t256, 0, st, active + first * n_blocks, flags,
                               (uint8_t)0);
            CDQ_LAUNCH_CHECK();
        }
        {
            const int64_t items = (int64_t)(n_gamma - first) * d_out > n_blocks ? (int64_t)(n_gamma - first) * d_out : n_blocks;
            hipLaunchKernelGGL(owc_flags_kernel, dim3((unsigned)((items + 255) / 256)), t256, 0, st, (const uint8_t*)cand, d_out, n_gamma,
                               first, block_rows, n_blocks, (const int32_t*)total, active, rows_active);
            CDQ_LAUNCH_CHECK();
        }
        hipLaunchKernelGGL(owc_row_residual_kernel, cols, t256, 0, st, Wt, d_in, bits, (const float*)lo, (const float*)hi, n_gamma,
                           (const int32_t*)row_col, (const uint8_t*)row_k, (const int32_t*)total, Wc);
        CDQ_LAUNCH_CHECK();
        rc = loss_launch(H, Wc, zeros, zeros, trial_q, d_out, d_in, d_in, row_loss, nullptr, loss_ws, loss_ws_bytes, st, rows_active);
        if (rc != CDQ_OK) return rc;
        hipLaunchKernelGGL(owc_update_best_rows_kernel, col_blocks, t256, 0, st, (const double*)row_loss, (const uint8_t*)row_k,
                           (const int32_t*)extras, (const int32_t*)base, cap, n_gamma, d_out, best_loss, best_gamma);
        CDQ_LAUNCH_CHECK();
        // 4. ... and what did not fit the rows (more candidates than columns: only when many columns fail the check), rank by
        // rank; idle launches otherwise
        for (int r = 1; r < n_gamma; ++r) {
            rc = rank_pass(r);
            if (rc != CDQ_OK) return rc;
        }
        if (researched != nullptr) CDQ_HIP_CHECK(hipMemcpyAsync(researched, count, sizeof(int32_t), hipMemcpyDeviceToDevice, st));
    } else {
    if (researched != nullptr) {            // the exhaustive search needs no check
        hipLaunchKernelGGL(owc_fill_f32_kernel, dim3(1), t256, 0, st, (float*)researched, (int64_t)1, 0.0f);
        CDQ_LAUNCH_CHECK();
    }
    for (int k = 1; k <= n_gamma; ++k) {
        const float gamma = (float)k / (float)n_gamma;
        hipLaunchKernelGGL(owc_quantize_kernel, cols, t256, 0, st, Wt, d_in, bits, lo, hi, gamma, (const float*)nullptr, trial_scale,
                           (float*)nullptr, trial_q);
        CDQ_LAUNCH_CHECK();
        const int rc = loss_launch(H, Wt, trial_scale, lo, trial_q, d_out, d_in, d_in, trial_loss, nullptr, loss_ws, loss_ws_bytes, st);
        if (rc != CDQ_OK) return rc;
        hipLaunchKernelGGL(owc_update_best_kernel, dim3((unsigned)((d_out + 255) / 256)), t256, 0, st, trial_loss, d_out, gamma,
                           k == 1 ? 1 : 0, best_loss, best_gamma);
        CDQ_LAUNCH_CHECK();
    }
    }
    hipLaunchKernelGGL(owc_quantize_kernel, cols, t256, 0, st, Wt, d_in, bits, lo, hi, 1.0f, best_gamma, scale, zero, Q);
    CDQ_LAUNCH_CHECK();
    if (G_out != nullptr) {
        if (!g_from_first_pass) {
            const int rc = gradient_launch(H, Wt, scale, zero, Q, d_out, d_in, d_in, G_out, st);
            if (rc != CDQ_OK) return rc;
        } else {
            // rows of the columns that ended at another grid point than their best-screened one, gathered as minus-residuals
            // (the same bits as the residual of scale, zero, Q) and multiplied again into their place
            const int block_rows = loss_block_rows();
            const int64_t n_blocks = (d_out + block_rows - 1) / block_rows;
            hipLaunchKernelGGL(owc_changed_kernel, col_blocks, t256, 0, st, (const float*)best_gamma, (const float*)first_gamma, d_out, g_changed);
            CDQ_LAUNCH_CHECK();
            hipLaunchKernelGGL(owc_scan_extras_kernel, dim3(1), dim3(1024), 0, st, (const int32_t*)g_changed, d_out, g_base, g_total);
            CDQ_LAUNCH_CHECK();
            hipLaunchKernelGGL(owc_changed_rows_kernel, col_blocks, t256, 0, st, (const int32_t*)g_changed, (const int32_t*)g_base,
                               (const float*)best_gamma, n_gamma, d_out, g_row_col, g_row_k, g_total);
            CDQ_LAUNCH_CHECK();
            hipLaunchKernelGGL(owc_row_blocks_kernel, dim3((unsigned)((n_blocks + 255) / 256)), t256, 0, st, (const int32_t*)g_total, block_rows,
                               n_blocks, g_rows_active);
            CDQ_LAUNCH_CHECK();
            hipLaunchKernelGGL(owc_row_residual_kernel, cols, t256, 0, st, Wt, d_in, bits, (const float*)lo, (const float*)hi, n_gamma,
                               (const int32_t*)g_row_col, (const uint8_t*)g_row_k, (const int32_t*)g_total, g_Wc);
            CDQ_LAUNCH_CHECK();
            const int rc = gradient_loss_launch(H, g_Wc, g_zeros, g_zeros, trial_q, d_out, d_in, d_in, G_out, nullptr, nullptr, 0, st,
                                                g_rows_active, g_row_col, g_total);
            if (rc != CDQ_OK) return rc;
        }
    }
    if (gamma_out != nullptr) CDQ_HIP_CHECK(hipMemcpyAsync(gamma_out, best_gamma, (size_t)d_out * sizeof(float), hipMemcpyDeviceToDevice, st));
    if (loss_out != nullptr) CDQ_HIP_CHECK(hipMemcpyAsync(loss_out, best_loss, (size_t)d_out * sizeof(double), hipMemcpyDeviceToDevice, st));
    return CDQ_OK;
}

}  // namespace cdq
