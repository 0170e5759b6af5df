/*
 * mkq_tuning.h -- tuning interface of libmkq: the linears of mkq.h with the kernel configuration chosen by
 * the caller instead of by the library.  Not needed to use the library; benchmarks sweep it and tests use it
 * to reach every kernel variant at small sizes and to check the library's own choice against the others.
 * Nothing here keeps state: the choice is an argument of the call.
 */
#ifndef MKQ_TUNING_H
#define MKQ_TUNING_H

#include "mkq.h"

#ifdef __cplusplus
extern "C" {
#endif

/* mkq_linear_int4 (section 3.1 Eq. 1 and the linears of section 3.2; same arguments, same results) with
 *   config    -1 = the library's choice; otherwise one kernel configuration by number:
 *             2, 3         register-staged generic kernel, 128x128 / 64x64 tiles (any K % 32 == 0)
 *             11 .. 29     ring kernel tile shapes (K % 128 == 0): 11 256x256/8 waves, 12 128x128 four-stage,
 *                          14 64x64 eight-stage, 18 256x128, 19 128x256, 20 256x128 with 32-byte stages,
 *                          27 64x64, 28 128x64, 29 128x128 three-stage
 *             31, 33, 35   ring kernel with K split between two wave groups of a workgroup (K % 256 == 0):
 *                          64x64 four-stage, 64x64 three-stage, 128x128
 *             30           first few-token kernel (M <= 128, K % 256 == 0; waves split K, operands through registers)
 *             50           few-token weight-streaming kernel (M <= 128, K % 256 == 0)
 *             60, 61, 62   128 x 128, 64 x 64 (two wave groups) and 128 x 64 tiles with the k loop also split
 *                          across workgroups (needs epi->splitk_scratch; k_slices must divide K's 128-code
 *                          stages and leave two per slice; measured slower than the unsplit tiles, kept for study)
 *   k_slices  0 = the library's choice; otherwise the number of K slices across workgroups of configurations
 *             50 (needs epi->splitk_scratch; clamped to what K and the scratch area allow) and 60 .. 62
 * A configuration that does not apply to the arguments returns MKQ_ERR_UNSUPPORTED before anything is enqueued. */
int mkq_tuning_linear_int4(const void *a, int a_dtype, float s_x, const uint8_t *Wq, const float *s_w,
                           const float *bias, int64_t M, int64_t N, int64_t K, void *out, int out_dtype,
                           const mkq_epilogue *epi, void *workspace, size_t workspace_bytes, void *stream,
                           int config, int k_slices);

/* mkq_linear_int4_stream with the number of 256-code stages that a wave keeps in flight (0 = the library's
 * choice; 2, 3, 4 or 6) and the number of K slices across workgroups (0 = the library's choice). */
int mkq_tuning_linear_int4_stream(const void *a, int a_dtype, float s_x, const uint8_t *Wq_stream, const float *s_w,
                                  const float *bias, int64_t M, int64_t N, int64_t K, void *out, int out_dtype,
                                  const mkq_epilogue *epi, void *workspace, size_t workspace_bytes, void *stream,
                                  int prefetch_stages, int k_slices);

/* mkq_linear_int8 with config -1 (the library's choice), 18 (256x128 tiles), 29 (128x128), 28 (128x64), 27 (64x64)
 * or 30 (few-token weight-streaming kernel: M <= 64, K % 128 == 0). */
int mkq_tuning_linear_int8(const int8_t *a, float s_x, const int8_t *Wq, const float *s_w, const float *bias,
                           int64_t M, int64_t N, int64_t K, void *out, int out_dtype, const mkq_epilogue *epi,
                           void *stream, int config);

/* mkq_linear_int4_e3m2 with config -1 (the library's choice), 41 (256x256 tiles, eight waves) or
 * 42 (256x128 tiles, four waves, two workgroups per compute unit). */
int mkq_tuning_linear_int4_e3m2(const uint8_t *a, float s_x, const uint8_t *Wq, const float *s_w,
                                const float *bias, int64_t M, int64_t N, int64_t K, void *out, int out_dtype,
                                const mkq_epilogue *epi, void *stream, int config);

/* Measured ceilings, printed by the benchmark beside every roofline fraction (they compute nothing of the
 * method).  All enqueue one kernel on `stream`; the caller times it.
 *   mkq_measure_stream    kind 0: read `bytes` from src (dst: 16 bytes, never written in practice), 1: write
 *                         `bytes` to dst, 2: copy src -> dst.  bytes % 16 == 0.  Device pointers, 16-byte aligned.
 *   mkq_measure_mfma_i8   a register-only loop of v_mfma_i32_32x32x32_i8, 8 independent accumulator tiles per
 *                         wave, two workgroups of four waves per compute unit, `iters` rounds; the operands
 *                         (6 x 16 bytes per lane) are read once from `operands`, which the caller fills with bytes
 *                         of the kind the GEMM multiplies (16 * code) -- the chip's clock under a matrix load
 *                         depends on the data.  mkq_measure_mfma_i8_operand_bytes() = the size it reads;
 *                         mkq_measure_mfma_i8_ops(iters) = integer operations of one launch (0 on error).
 * Errors: NULL, ALIGN, SHAPE, DTYPE (kind), WORKSPACE (operands too small), HIP. */
int mkq_measure_stream(int kind, const void *src, void *dst, size_t bytes, void *stream);
size_t mkq_measure_mfma_i8_operand_bytes(void);
int64_t mkq_measure_mfma_i8_ops(int iters);
int mkq_measure_mfma_i8(const void *operands, size_t operand_bytes, int iters, void *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MKQ_TUNING_H */
