// Internal declarations shared by the translation units of libcdq (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "cdq.h"

#define CDQ_HIP_CHECK(expr)                         \
    do {                                            \
        hipError_t cdq_err_ = (expr);               \
        if (cdq_err_ != hipSuccess) return CDQ_EHIP; \
    } while (0)

#define CDQ_LAUNCH_CHECK() CDQ_HIP_CHECK(hipGetLastError())

static inline size_t cdq_align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

namespace cdq {

// ---- hessian.hip
size_t hessian_workspace_bytes(int64_t n, int64_t d_in);
int hessian_launch(const void* X, int x_dtype, int64_t n, int64_t d_in, float* H, int accumulate,
                   float lambda_rel, void* ws, size_t ws_bytes, hipStream_t st);

// ---- rtn.hip
int rtn_launch(const float* Wt, int64_t d_out, int64_t d_in, int bits, int64_t group,
               float* scale, float* zero, uint8_t* Q, hipStream_t st);

// ---- eh_gemm.hip : C = E * H with fp64 accumulation; epilogue stores G or row partial losses
size_t loss_workspace_bytes(int64_t d_out, int64_t d_in);
int gradient_launch(const float* H, const float* Wt, const float* scale, const float* zero,
                    const uint8_t* Q, int64_t d_out, int64_t d_in, int64_t group, float* G, hipStream_t st,
                    double* G64 = nullptr);   // G64 non-null: store the fp64 sums there instead of G
int loss_launch(const float* H, const float* Wt, const float* scale, const float* zero, const uint8_t* Q,
                int64_t d_out, int64_t d_in, int64_t group, double* loss_per_col, double* loss_total,
                void* ws, size_t ws_bytes, hipStream_t st, const uint8_t* row_block_active = nullptr);
// row_block_active non-null: one byte per block of loss_block_rows() columns of W; blocks with a zero are skipped and
// their entries of loss_per_col are unspecified
// The product G = E H and, from the same fp64 sums, each row's loss (loss_per_col NULL: product only; else ws as for
// loss_launch).  row_map / n_rows_dev (both or neither): operand row s < *n_rows_dev is written to row row_map[s] of G, the
// other rows are not written.
int gradient_loss_launch(const float* H, const float* Wt, const float* scale, const float* zero, const uint8_t* Q,
                         int64_t d_out, int64_t d_in, int64_t group, float* G, double* loss_per_col, void* ws, size_t ws_bytes,
                         hipStream_t st, const uint8_t* row_block_active, const int32_t* row_map, const int32_t* n_rows_dev);
int loss_block_rows();
int loss_static_launch(const float* H, const float* Wt, const float* scale, const float* zero, const uint8_t* Q,
                       int64_t d_out, int64_t d_in, int64_t group, double* loss_per_col, double* loss_total, hipStream_t st);

// ---- owc_screen.hip : every clipping strength evaluated in bf16 first, candidates ranked per column
bool owc_screen_applies(int64_t d_out, int64_t d_in, int n_gamma);
size_t owc_screen_workspace_bytes(int64_t d_out, int64_t d_in, int n_gamma, int64_t n_blocks);
int owc_screen_launch(const float* H, const float* Wt, int64_t d_out, int64_t d_in, int bits, int n_gamma, const float* lo, const float* hi,
                      float margin, int block_rows, int64_t n_blocks, void* ws, uint8_t** cand_out, uint8_t** active_out,
                      const float** screened_out, hipStream_t st);

// ---- owc.hip
size_t owc_workspace_bytes(int64_t d_out, int64_t d_in);
int owc_launch(const float* H, const float* Wt, int64_t d_out, int64_t d_in, int bits, int n_gamma, float screen_margin, float* scale,
               float* zero, uint8_t* Q, float* gamma_out, double* loss_out, int32_t* researched, float* G_out, void* ws, size_t ws_bytes,
               hipStream_t st);

// ---- owc_cd.hip
int owc_cd_launch(const float* H, const float* Wt, int64_t d_out, int64_t d_in, int bits, int64_t group, int n_gamma, int64_t T,
                  float* scale, float* zero, uint8_t* Q, int32_t* gamma_idx, int32_t* moves, int32_t* trace, int64_t trace_cap,
                  void* ws, size_t ws_bytes, bool force_simple, hipStream_t st);
size_t owc_cd_workspace_bytes(int64_t d_out, int64_t d_in);

// ---- bcd.hip
size_t bcd_workspace_bytes(int64_t d_out, int64_t d_in, int64_t T);
int bcd_launch(const float* H, const float* Wt, const float* scale, const float* zero, uint8_t* Q, int64_t d_out, int64_t d_in,
               int bits, int64_t group, const int32_t* parts, int64_t T, int32_t* moves, float* G_out, int32_t* trace,
               int64_t trace_cap, int flags, void* ws, size_t ws_bytes, hipStream_t st);

// ---- cyclic.hip
size_t cyclic_workspace_bytes(int64_t d_out, int64_t d_in);
int cyclic_launch(const float* H, const float* Wt, const float* scale, const float* zero, uint8_t* Q, int64_t d_out, int64_t d_in,
                  int bits, int64_t group, int64_t T, cdq_col_stats* stats, float* G_out, int32_t* trace, int64_t trace_cap,
                  void* ws, size_t ws_bytes, hipStream_t st);

// ---- stepwise.hip
int score_argmin_launch(const float* hdiag, const float* scale, const uint8_t* Q, const float* G, int64_t d_out, int64_t d_in,
                        int bits, int64_t group, int32_t* out_i, int32_t* out_r, float* out_s, hipStream_t st);
int gather_update_launch(const float* H, const float* scale, uint8_t* Q, float* G, int64_t d_out, int64_t d_in, int64_t group,
                         const int32_t* sel_i, const int32_t* sel_r, int32_t* moves, hipStream_t st);

// ---- cd_fused.hip
int cd_choose_shape(int64_t d_out, int64_t d_in, int64_t group, bool aligned16, int* waves, int* elems, int* vec);
int cd_choose_teams(int64_t d_out, int waves, int elems, int vec);       // columns resident per compute unit: 1 or 2
int cd_launch(const float* H, const float* hdiag, float* G0, const float* scale, uint8_t* Q,          // G0 is overwritten
              int64_t d_out, int64_t d_in, int bits, int64_t group, int64_t T, cdq_col_stats* stats,
              int waves, int elems, int vec, int exact_only, int32_t* trace, int64_t trace_cap, float* G_out,
              hipStream_t st, int teams_per_cu = 0);      // 0: choose; 2 only for 16 wavefronts x 16 per lane, 16-byte chunks
int extract_diag_launch(const float* H, int64_t d_in, float* hdiag, hipStream_t st);

}  // namespace cdq
