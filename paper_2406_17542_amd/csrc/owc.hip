// Optimal Weight Clipping (paper Section 3.1, "Initializing a, b, q"; Eq. (2)): per output column,
// grid search over the clipping strength gamma for the smallest layer loss of Eq. (1).
//   b = min w,  a(gamma) = gamma (max w - min w)/(2^c - 1),  q = clamp(round((w - b)/a), 0, 2^c - 1)
// The grid is gamma_k = k/n_gamma, k = 1..n_gamma (gamma = 1 is MinMax; equal losses keep the
// larger gamma).  Each gamma costs one pass of the fp64 loss kernel over all columns.
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

}  // namespace

size_t owc_workspace_bytes(int64_t d_out, int64_t d_in) {
    size_t b = 0;
    b += cdq_align_up((size_t)d_out * sizeof(float), 256) * 4;       // lo, hi, trial scale, best gamma
    b += cdq_align_up((size_t)d_out * sizeof(double), 256) * 2;      // trial loss, best loss
    b += cdq_align_up((size_t)d_out * d_in, 256);                    // trial codes
    b += loss_workspace_bytes(d_out, d_in);
    return b;
}

int owc_launch(const float* H, const float* Wt, int64_t d_out, int64_t d_in, int bits, int n_gamma, float* scale, float* zero,
               uint8_t* Q, float* gamma_out, double* loss_out, void* ws, size_t ws_bytes, hipStream_t st) {
    if (d_out == 0) return CDQ_OK;
    if (ws == nullptr || ((uintptr_t)ws & 255) || ws_bytes < owc_workspace_bytes(d_out, d_in)) return CDQ_EWORKSPACE;
    if (d_out > 0x7fffffffLL) return CDQ_EUNSUPPORTED;
    char* p = (char*)ws;
    const size_t fsz = cdq_align_up((size_t)d_out * sizeof(float), 256), dsz = cdq_align_up((size_t)d_out * sizeof(double), 256);
    float* lo = (float*)p; p += fsz;
    float* hi = (float*)p; p += fsz;
    float* trial_scale = (float*)p; p += fsz;
    float* best_gamma = (float*)p; p += fsz;
    double* trial_loss = (double*)p; p += dsz;
    double* best_loss = (double*)p; p += dsz;
    uint8_t* trial_q = (uint8_t*)p; p += cdq_align_up((size_t)d_out * d_in, 256);
    void* loss_ws = p;
    const size_t loss_ws_bytes = loss_workspace_bytes(d_out, d_in);
    const dim3 cols((unsigned)d_out), t256(256);

    hipLaunchKernelGGL(owc_minmax_kernel, cols, t256, 0, st, Wt, d_in, lo, hi);
    CDQ_LAUNCH_CHECK();
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
    hipLaunchKernelGGL(owc_quantize_kernel, cols, t256, 0, st, Wt, d_in, bits, lo, hi, 1.0f, best_gamma, scale, zero, Q);
    CDQ_LAUNCH_CHECK();
    if (gamma_out != nullptr) CDQ_HIP_CHECK(hipMemcpyAsync(gamma_out, best_gamma, (size_t)d_out * sizeof(float), hipMemcpyDeviceToDevice, st));
    if (loss_out != nullptr) CDQ_HIP_CHECK(hipMemcpyAsync(loss_out, best_loss, (size_t)d_out * sizeof(double), hipMemcpyDeviceToDevice, st));
    return CDQ_OK;
}

}  // namespace cdq
