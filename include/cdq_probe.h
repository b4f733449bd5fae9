/*
 * libcdq measurement helpers -- not part of the method.  Plain memory and matrix-core loops that
 * give the "achievable" figures a benchmark quotes beside the kernels of cdq.h (the paper attributes
 * the cost of coordinate descent to gathers, appendix "Runtime Analysis"), and a copy of known size
 * against which hardware byte counters are scaled.  Same conventions as cdq.h: device pointers owned
 * by the caller, `stream` a hipStream_t passed as void*, calls only enqueue, negative error codes.
 */
#ifndef CDQ_PROBE_H
#define CDQ_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 *   cdq_probe_copy    dst[0..bytes) = src[0..bytes)  (reads `bytes`, writes `bytes`; % 16 == 0)
 *   cdq_probe_read    streams `bytes` once; *sink is scratch (one float), practically never written
 *   cdq_probe_gather  `teams` groups of `waves_per_row` wavefronts each read `iters` pseudo-random
 *                     rows of `row_bytes` from a matrix of `n_rows` rows: the loop's access
 *                     pattern without its arithmetic.
 */
int cdq_probe_copy(const void *src, void *dst, size_t bytes, void *stream);
int cdq_probe_read(const void *src, size_t bytes, float *sink, void *stream);
int cdq_probe_gather(const void *H, int64_t n_rows, int64_t row_bytes, int64_t teams, int waves_per_row,
                     int64_t iters, float *sink, void *stream);
/* Matrix-core-only loop, no memory traffic: kind 0 = v_mfma_f32_32x32x16_bf16 on constant operands (8 wavefronts
 * per block, 8 independent MFMAs per round), kind 1 = v_mfma_f64_16x16x4_f64 (16 wavefronts per block, 4 per round),
 * kind 2 = v_mfma_f32_32x32x16_bf16 on pseudo-random operands (4 wavefronts per block, 32 MFMAs per round): the power
 * the matrix cores draw, and with it the clock the chip holds, depends on the operand bits, so kind 2 is the ceiling for
 * a GEMM on real data and kind 0 the ceiling of the instruction rate;
 * `blocks` workgroups each run `iters` rounds.  *flop (host pointer, may be NULL) receives the operation count of
 * the launch.  Timed by the benchmark: the ceiling the GEMM kernels are compared with on this machine. */
int cdq_probe_mfma(int kind, int64_t blocks, int64_t iters, float *sink, double *flop, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CDQ_PROBE_H */
