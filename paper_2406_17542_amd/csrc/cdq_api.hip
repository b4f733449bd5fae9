// C ABI of libcdq: argument checks, workspace layout, dispatch.  See include/cdq.h.
#include "cdq_internal.h"

namespace {

bool bad_bits(int bits) { return bits < 2 || bits > 4; }
bool bad_layer(int64_t d_out, int64_t d_in, int64_t group) {
    return d_out < 0 || d_in <= 0 || group <= 0 || group > d_in || d_in % group != 0;
}
bool misaligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) != 0; }

size_t cd_workspace_bytes(int64_t d_out, int64_t d_in) {
    // G0 [d_out][d_in], diag(H) [d_in], and three per-column arrays used by the stepwise path
    return cdq_align_up((size_t)d_out * d_in * sizeof(float), 256) + cdq_align_up((size_t)d_in * sizeof(float), 256) +
           3 * cdq_align_up((size_t)d_out * sizeof(int32_t), 256);
}

}  // namespace

extern "C" {

const char* cdq_strerror(int code) {
    switch (code) {
        case CDQ_OK: return "ok";
        case CDQ_EINVAL: return "invalid argument (null pointer, bad shape, bits not in {2,3,4}, d_in % group != 0, misaligned data)";
        case CDQ_EWORKSPACE: return "workspace missing, not 256-byte aligned, or smaller than cdq_workspace_bytes()";
        case CDQ_EHIP: return "HIP runtime error";
        case CDQ_EUNSUPPORTED: return "shape outside what the kernels cover";
        default: return "unknown cdq error code";
    }
}

size_t cdq_workspace_bytes(int op, int64_t n, int64_t d_out, int64_t d_in) {
    if (d_in <= 0 || d_out < 0) return 0;
    switch (op) {
        case CDQ_OP_HESSIAN: return cdq::hessian_workspace_bytes(n, d_in);
        case CDQ_OP_GREEDY_CD: return cd_workspace_bytes(d_out, d_in);
        case CDQ_OP_LOSS: return cdq::loss_workspace_bytes(d_out, d_in);
        case CDQ_OP_INIT_OWC: return cdq::owc_workspace_bytes(d_out, d_in);
        case CDQ_OP_INIT_OWC_CD: return cdq::owc_cd_workspace_bytes(d_out, d_in);
        case CDQ_OP_BCD: return cdq::bcd_workspace_bytes(d_out, d_in, n);
        case CDQ_OP_CYCLIC_CD: return cdq::cyclic_workspace_bytes(d_out, d_in);
        default: return 0;
    }
}

int cdq_hessian(const void* X, int x_dtype, int64_t n, int64_t d_in, float* H, int accumulate, float lambda_rel,
                void* workspace, size_t workspace_bytes, void* stream) {
    if (X == nullptr || H == nullptr || n < 0 || d_in <= 0) return CDQ_EINVAL;
    if (x_dtype != CDQ_F32 && x_dtype != CDQ_BF16) return CDQ_EINVAL;
    if (!(lambda_rel >= 0.0f)) return CDQ_EINVAL;
    if (x_dtype == CDQ_BF16 && (d_in % 8 != 0 || misaligned(X, 16))) return CDQ_EINVAL;
    if (x_dtype == CDQ_F32 && (d_in % 4 != 0 || misaligned(X, 16))) return CDQ_EINVAL;
    if (misaligned(H, 16)) return CDQ_EINVAL;
    return cdq::hessian_launch(X, x_dtype, n, d_in, H, accumulate != 0, lambda_rel, workspace, workspace_bytes,
                               (hipStream_t)stream);
}

int cdq_init_rtn(const float* Wt, int64_t d_out, int64_t d_in, int bits, int64_t group, float* scale, float* zero,
                 uint8_t* Q, void* stream) {
    if (bad_bits(bits) || bad_layer(d_out, d_in, group)) return CDQ_EINVAL;
    if (d_out == 0) return CDQ_OK;        // empty layer: nothing to write, pointers may be null
    if (Wt == nullptr || scale == nullptr || zero == nullptr || Q == nullptr) return CDQ_EINVAL;
    return cdq::rtn_launch(Wt, d_out, d_in, bits, group, scale, zero, Q, (hipStream_t)stream);
}

int cdq_init_owc(const float* H, const float* Wt, int64_t d_out, int64_t d_in, int bits, int64_t group, int n_gamma,
                 float screen_margin, float* scale, float* zero, uint8_t* Q, float* gamma_out, double* loss_out,
                 int32_t* researched, float* G_out, void* workspace, size_t workspace_bytes, void* stream) {
    if (bad_bits(bits) || bad_layer(d_out, d_in, group) || n_gamma < 1 || n_gamma > 4096) return CDQ_EINVAL;
    if (!(screen_margin >= 0.0f) || screen_margin > 1.0f) return CDQ_EINVAL;
    if (group != d_in) return CDQ_EUNSUPPORTED;       // Eq. (2) has one clipping strength per column
    if (d_out == 0) return CDQ_OK;
    if (H == nullptr || Wt == nullptr || scale == nullptr || zero == nullptr || Q == nullptr) return CDQ_EINVAL;
    return cdq::owc_launch(H, Wt, d_out, d_in, bits, n_gamma, screen_margin, scale, zero, Q, gamma_out, loss_out, researched, G_out,
                           workspace, workspace_bytes, (hipStream_t)stream);
}

int cdq_init_owc_cd(const float* H, const float* Wt, int64_t d_out, int64_t d_in, int bits, int64_t group, int n_gamma,
                    int64_t T, float* scale, float* zero, uint8_t* Q, int32_t* gamma_idx, int32_t* moves, int32_t* trace,
                    int64_t trace_cap, int variant, void* workspace, size_t workspace_bytes, void* stream) {
    if (bad_bits(bits) || bad_layer(d_out, d_in, group) || n_gamma < 1 || T < 0 || variant < 0 || variant > 1) return CDQ_EINVAL;
    if (trace != nullptr && trace_cap <= 0) return CDQ_EINVAL;
    if (d_out == 0) return CDQ_OK;
    if (H == nullptr || Wt == nullptr || scale == nullptr || zero == nullptr || Q == nullptr) return CDQ_EINVAL;
    return cdq::owc_cd_launch(H, Wt, d_out, d_in, bits, group, n_gamma, T, scale, zero, Q, gamma_idx, moves, trace, trace_cap,
                              workspace, workspace_bytes, variant == 1, (hipStream_t)stream);
}

int cdq_bcd(const float* H, const float* Wt, const float* scale, const float* zero, uint8_t* Q, int64_t d_out, int64_t d_in,
            int bits, int64_t group, int k, const int32_t* parts, int64_t T, int32_t* moves, float* G_out, int32_t* trace,
            int64_t trace_cap, int flags, void* workspace, size_t workspace_bytes, void* stream) {
    if (bad_bits(bits) || bad_layer(d_out, d_in, group) || T < 0 || k < 1 || (flags & ~7) != 0) return CDQ_EINVAL;
    if (trace != nullptr && trace_cap <= 0) return CDQ_EINVAL;
    if (k != 2) return CDQ_EUNSUPPORTED;              // k = 1 is cdq_greedy_cd; larger blocks are not built
    if (d_in % 2 != 0) return CDQ_EINVAL;
    if (d_out == 0) return CDQ_OK;
    if (H == nullptr || Wt == nullptr || scale == nullptr || zero == nullptr || Q == nullptr) return CDQ_EINVAL;
    if (T > 0 && parts == nullptr) return CDQ_EINVAL;
    return cdq::bcd_launch(H, Wt, scale, zero, Q, d_out, d_in, bits, group, parts, T, moves, G_out, trace, trace_cap, flags,
                           workspace, workspace_bytes, (hipStream_t)stream);
}

int cdq_cyclic_cd(const float* H, const float* Wt, const float* scale, const float* zero, uint8_t* Q, int64_t d_out, int64_t d_in,
                  int bits, int64_t group, int64_t T, cdq_col_stats* stats, float* G_out, int32_t* trace, int64_t trace_cap,
                  void* workspace, size_t workspace_bytes, void* stream) {
    if (bad_bits(bits) || bad_layer(d_out, d_in, group) || T < 0) return CDQ_EINVAL;
    if (trace != nullptr && trace_cap <= 0) return CDQ_EINVAL;
    if (d_out == 0) return CDQ_OK;
    if (H == nullptr || Wt == nullptr || scale == nullptr || zero == nullptr || Q == nullptr) return CDQ_EINVAL;
    return cdq::cyclic_launch(H, Wt, scale, zero, Q, d_out, d_in, bits, group, T, stats, G_out, trace, trace_cap, workspace,
                              workspace_bytes, (hipStream_t)stream);
}

int cdq_gradient(const float* H, const float* Wt, const float* scale, const float* zero, const uint8_t* Q,
                 int64_t d_out, int64_t d_in, int64_t group, float* G, void* stream) {
    if (bad_layer(d_out, d_in, group)) return CDQ_EINVAL;
    if (d_out == 0) return CDQ_OK;
    if (H == nullptr || Wt == nullptr || scale == nullptr || zero == nullptr || Q == nullptr || G == nullptr) return CDQ_EINVAL;
    return cdq::gradient_launch(H, Wt, scale, zero, Q, d_out, d_in, group, G, (hipStream_t)stream);
}

int cdq_greedy_cd_ex(const float* H, const float* Wt, const float* scale, const float* zero, uint8_t* Q,
                     int64_t d_out, int64_t d_in, int bits, int64_t group, int64_t T, cdq_col_stats* stats,
                     const cdq_cd_options* opts, void* workspace, size_t workspace_bytes, void* stream) {
    if (bad_bits(bits) || bad_layer(d_out, d_in, group) || T < 0) return CDQ_EINVAL;
    if (d_out == 0) return CDQ_OK;
    if (H == nullptr || Wt == nullptr || scale == nullptr || zero == nullptr || Q == nullptr) return CDQ_EINVAL;
    if (d_in > CDQ_MAX_D_IN) return CDQ_EUNSUPPORTED;
    if (opts != nullptr && opts->trace != nullptr && opts->trace_cap <= 0) return CDQ_EINVAL;
    int waves = 0, elems = 0, vec = 0;
    // the shape is chosen for the vector width the pointers allow: a misaligned layer gets a scalar-load shape
    int rc = cdq::cd_choose_shape(d_out, d_in, group, !(misaligned(Q, 4) || misaligned(H, 16)), &waves, &elems, &vec);
    if (rc != CDQ_OK) return rc;
    if (opts != nullptr && (opts->waves_per_column != 0 || opts->elems_per_lane != 0)) {
        const int w = opts->waves_per_column, e = opts->elems_per_lane;
        const bool w_ok = (w == 1 || w == 2 || w == 4 || w == 8 || w == 16);
        const bool e_ok = (e == 4 || e == 8 || e == 16 || e == 32 || ((e == 24 || e == 36) && w == 16));
        if (!w_ok || !e_ok || (int64_t)64 * w * e < d_in) return CDQ_EINVAL;
        waves = w;
        elems = e;
    }
    if ((elems == 36 || elems == 24) && vec != 4) return CDQ_EUNSUPPORTED;      // the kernel with the Hessian diagonal in LDS takes 16-byte chunks only
    hipStream_t st = (hipStream_t)stream;
    float *G0, *hdiag;
    if (opts != nullptr && opts->G0 != nullptr) {             // the caller brings the start gradient: only the diagonal needs room
        if (misaligned(opts->G0, 16)) return CDQ_EINVAL;
        if (workspace == nullptr || misaligned(workspace, 256) || workspace_bytes < cdq_align_up((size_t)d_in * sizeof(float), 256))
            return CDQ_EWORKSPACE;
        G0 = opts->G0;
        hdiag = (float*)workspace;
    } else {
        if (workspace == nullptr || misaligned(workspace, 256) || workspace_bytes < cd_workspace_bytes(d_out, d_in)) return CDQ_EWORKSPACE;
        G0 = (float*)workspace;
        hdiag = (float*)((char*)workspace + cdq_align_up((size_t)d_out * d_in * sizeof(float), 256));
        rc = cdq::gradient_launch(H, Wt, scale, zero, Q, d_out, d_in, group, G0, st);
        if (rc != CDQ_OK) return rc;
    }
    rc = cdq::extract_diag_launch(H, d_in, hdiag, st);
    if (rc != CDQ_OK) return rc;
    if (opts != nullptr && opts->ev_loop_begin != nullptr) CDQ_HIP_CHECK(hipEventRecord((hipEvent_t)opts->ev_loop_begin, st));
    rc = cdq::cd_launch(H, hdiag, G0, scale, Q, d_out, d_in, bits, group, T, stats, waves, elems, vec,
                        (opts != nullptr && opts->exact_scorer_only) ? 1 : 0, opts ? opts->trace : nullptr, opts ? opts->trace_cap : 0, opts ? opts->G_out : nullptr, st,
                        opts ? opts->teams_per_cu : 0);
    if (rc != CDQ_OK) return rc;
    if (opts != nullptr && opts->ev_loop_end != nullptr) CDQ_HIP_CHECK(hipEventRecord((hipEvent_t)opts->ev_loop_end, st));
    return CDQ_OK;
}

int cdq_greedy_cd_shape(int64_t d_out, int64_t d_in, int64_t group, int aligned16, int32_t* waves_per_column,
                        int32_t* elems_per_lane, int32_t* teams_per_cu) {
    if (bad_layer(d_out, d_in, group) || waves_per_column == nullptr || elems_per_lane == nullptr) return CDQ_EINVAL;
    if (d_in > CDQ_MAX_D_IN) return CDQ_EUNSUPPORTED;
    int waves = 0, elems = 0, vec = 0;
    const int rc = cdq::cd_choose_shape(d_out, d_in, group, aligned16 != 0, &waves, &elems, &vec);
    if (rc != CDQ_OK) return rc;
    *waves_per_column = waves;
    *elems_per_lane = elems;
    if (teams_per_cu != nullptr) *teams_per_cu = cdq::cd_choose_teams(d_out, waves, elems, vec);
    return CDQ_OK;
}

int cdq_score_argmin(const float* Hdiag, const float* scale, const uint8_t* Q, const float* G, int64_t d_out, int64_t d_in,
                     int bits, int64_t group, int32_t* best_i, int32_t* best_r, float* best_s, void* stream) {
    if (bad_bits(bits) || bad_layer(d_out, d_in, group)) return CDQ_EINVAL;
    if (d_out == 0) return CDQ_OK;
    if (Hdiag == nullptr || scale == nullptr || Q == nullptr || G == nullptr || best_i == nullptr || best_r == nullptr ||
        best_s == nullptr)
        return CDQ_EINVAL;
    return cdq::score_argmin_launch(Hdiag, scale, Q, G, d_out, d_in, bits, group, best_i, best_r, best_s, (hipStream_t)stream);
}

int cdq_gather_update(const float* H, const float* scale, uint8_t* Q, float* G, int64_t d_out, int64_t d_in, int64_t group,
                      const int32_t* best_i, const int32_t* best_r, int32_t* moves, void* stream) {
    if (bad_layer(d_out, d_in, group)) return CDQ_EINVAL;
    if (d_out == 0) return CDQ_OK;
    if (H == nullptr || scale == nullptr || Q == nullptr || G == nullptr || best_i == nullptr || best_r == nullptr) return CDQ_EINVAL;
    return cdq::gather_update_launch(H, scale, Q, G, d_out, d_in, group, best_i, best_r, moves, (hipStream_t)stream);
}

int cdq_greedy_cd_stepwise(const float* H, const float* Wt, const float* scale, const float* zero, uint8_t* Q, int64_t d_out,
                           int64_t d_in, int bits, int64_t group, int64_t T, int32_t* moves, void* workspace,
                           size_t workspace_bytes, void* stream) {
    if (bad_bits(bits) || bad_layer(d_out, d_in, group) || T < 0) return CDQ_EINVAL;
    if (d_out == 0) return CDQ_OK;
    if (H == nullptr || Wt == nullptr || scale == nullptr || zero == nullptr || Q == nullptr) return CDQ_EINVAL;
    const size_t g_bytes = cdq_align_up((size_t)d_out * d_in * sizeof(float), 256);
    const size_t h_bytes = cdq_align_up((size_t)d_in * sizeof(float), 256);
    const size_t c_bytes = cdq_align_up((size_t)d_out * sizeof(int32_t), 256);
    if (workspace == nullptr || misaligned(workspace, 256) || workspace_bytes < g_bytes + h_bytes + 3 * c_bytes) return CDQ_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    char* p = (char*)workspace;
    float* G = (float*)p; p += g_bytes;
    float* hdiag = (float*)p; p += h_bytes;
    int32_t* bi = (int32_t*)p; p += c_bytes;
    int32_t* br = (int32_t*)p; p += c_bytes;
    float* bs = (float*)p;
    int rc = cdq::gradient_launch(H, Wt, scale, zero, Q, d_out, d_in, group, G, st);
    if (rc != CDQ_OK) return rc;
    rc = cdq::extract_diag_launch(H, d_in, hdiag, st);
    if (rc != CDQ_OK) return rc;
    for (int64_t t = 0; t < T; ++t) {           // converged columns skip their update, so extra iterations are no-ops
        rc = cdq::score_argmin_launch(hdiag, scale, Q, G, d_out, d_in, bits, group, bi, br, bs, st);
        if (rc != CDQ_OK) return rc;
        rc = cdq::gather_update_launch(H, scale, Q, G, d_out, d_in, group, bi, br, moves, st);
        if (rc != CDQ_OK) return rc;
    }
    return CDQ_OK;
}

int cdq_greedy_cd(const float* H, const float* Wt, const float* scale, const float* zero, uint8_t* Q, int64_t d_out,
                  int64_t d_in, int bits, int64_t group, int64_t T, cdq_col_stats* stats, void* workspace,
                  size_t workspace_bytes, void* stream) {
    return cdq_greedy_cd_ex(H, Wt, scale, zero, Q, d_out, d_in, bits, group, T, stats, nullptr, workspace, workspace_bytes,
                            stream);
}

int cdq_loss(const float* H, const float* Wt, const float* scale, const float* zero, const uint8_t* Q, int64_t d_out,
             int64_t d_in, int64_t group, double* loss_per_col, double* loss_total, void* workspace,
             size_t workspace_bytes, void* stream) {
    if (bad_layer(d_out, d_in, group)) return CDQ_EINVAL;
    if (loss_per_col == nullptr && loss_total == nullptr) return CDQ_EINVAL;
    if (d_out > 0 && (H == nullptr || Wt == nullptr || scale == nullptr || zero == nullptr || Q == nullptr)) return CDQ_EINVAL;
    return cdq::loss_launch(H, Wt, scale, zero, Q, d_out, d_in, group, loss_per_col, loss_total, workspace, workspace_bytes,
                            (hipStream_t)stream);
}

int cdq_loss_static(const float* H, const float* Wt, const float* scale, const float* zero, const uint8_t* Q, int64_t d_out,
                    int64_t d_in, int64_t group, double* loss_per_col, double* loss_total, void* stream) {
    if (bad_layer(d_out, d_in, group)) return CDQ_EINVAL;
    if (loss_per_col == nullptr && loss_total == nullptr) return CDQ_EINVAL;
    if (d_out > 0 && (H == nullptr || Wt == nullptr || scale == nullptr || zero == nullptr || Q == nullptr)) return CDQ_EINVAL;
    return cdq::loss_static_launch(H, Wt, scale, zero, Q, d_out, d_in, group, loss_per_col, loss_total, (hipStream_t)stream);
}

}  // extern "C"
