/*
 * interlock_test.h - test and profiling hooks of libinterlock.  Not part of the training-step
 * boundary (interlock.h): these two calls exist so that tests and micro-benchmarks can reach single
 * kernels and per-kernel-class timings.  Same conventions: device pointers owned by the caller,
 * every function returns a status code or a count, nothing is printed.
 */
#ifndef INTERLOCK_TEST_H
#define INTERLOCK_TEST_H

#include "interlock.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Profiling (cfg.profile != 0): synchronises the stream and returns, per kernel class,
 * launches and total milliseconds since the last call, measured with HIP events recorded
 * on the library's stream before and after each launch group (`ms`; this includes the few
 * microseconds an event costs between launches), the algorithmic flops and bytes of those
 * launches, and for the bf16 GEMM classes `kernel_ms`: the execution time of the MFMA GEMM
 * kernels alone, from events attached to each dispatch (0 for the other classes).  With
 * cfg.profile == 1 everything runs on the caller's stream (no internal side stream); with
 * cfg.profile == 2 the step runs on both streams as it does unprofiled and only `kernel_ms`,
 * the launches, flops and bytes of the GEMM classes are filled (`ms` stays 0): the GEMM kernels'
 * durations inside the real step, other kernels running beside them.
 * `names` receives pointers to static strings; any output array may be NULL.  Returns the
 * number of classes written (<= cap), or a negative status code.
 */
int il_profile_read(il_ctx *ctx, int32_t cap, const char **names, int64_t *launches, double *ms,
                    double *flops, double *bytes, double *kernel_ms);

/*
 * Kernel-level test hook: one GEMM launch of the library's own kernels, outside any step, so
 * that tests and micro-benchmarks can reach each tile configuration and epilogue directly.
 *   C[M,N] = epilogue( sum_k A(m,k) B(k,n) )
 * dtype: il_dtype of A, B (and of C for the bf16/fp32-typed epilogues, see `epi`);
 * a_kmajor / b_kmajor: 0 = operand stored [rows, K] row-major, 1 = stored [K, rows] row-major;
 * epi: 0 store (T) | 1 +bias (T) | 2 +bias, C = pre-activation, C2 = GELU (T, T) |
 *      3 +bias +res (fp32 out) | 4 * GELU'(aux[row % aux_wrap]) (T) | 5 store fp32 |
 *      6 C = scale*acc (+ C if beta) (fp32) | 7 the head's logits tile (bf16 operands, forward layout only, not
 *      the 64x64 tiles): C = acc as IEEE half, clamped to the finite range; if C2 is given also the softmax
 *      statistics of the fp32 accumulators: C2 = fp32 [M][G][2], G = ceil(N / 64), (max, sum of exp(z - max)) of
 *      every group of 64 columns, followed by fp32 [M] target logits z[row, aux[row]] with aux = int32 [M]
 *      targets (rows whose target is outside [0, N) are left unwritten);
 * tile: 0 = library's choice, else (bf16 only; "+4" = four wavefronts that only load)
 *       1 = 256x256 / 8+4 wavefronts, 2 = 128x128 / 4+4, two K steps staged, 3 = 128x128 / 4+4, four staged,
 *       4 = 64x64 / 4 wavefronts, 5 = 64x64 / 4+4, four staged, 6 = 256x128 / 8+4, three staged,
 *       7 = 128x256 / 8+4, three staged, 8 = 256x256 / 8+4 as a persistent kernel (one workgroup per CU
 *       walks over its tiles; what the library itself uses for that tile).
 * All pointers are device pointers; unused ones may be NULL.  Returns an il_status.
 */
int il_test_gemm(int32_t dtype, const void *A, const void *B, int32_t M, int32_t N, int32_t K, int32_t lda,
                 int32_t ldb, int32_t a_kmajor, int32_t b_kmajor, int32_t epi, void *C, void *C2, int32_t ldc,
                 const void *bias, const float *res, const void *aux, int32_t aux_wrap, float scale,
                 int32_t beta, int32_t tile, void *stream);

/* ---- measured peaks of the board (reported beside the nominal 2.5 PFLOP/s and 8 TB/s) ------------- */

/*
 * Matrix-unit-only loop: 512 workgroups of four wavefronts, each issuing `iters` x 4 independent
 * v_mfma_f32_32x32x16_bf16 on register operands (no memory traffic), timed with HIP events on `stream`
 * (the call synchronises).  scratch: device, at least 1 KiB (never written in practice).
 * *tflops_out receives the achieved dense bf16 TFLOP/s.  IL_E_ARG for NULL pointers or iters outside
 * [1, 2^22].
 */
int il_measure_mfma_peak(float *scratch, int32_t iters, void *stream, double *tflops_out);

/*
 * Streaming copy dst[0..bytes) = src[0..bytes) in two forms, each run for `reps` launches after one
 * warm-up launch and timed with HIP events on `stream` (the call synchronises): `stream_copy_kernel`
 * (16 bytes per lane, plain loads and stores) and `stream_copy4_kernel` (four 16-byte vectors in flight
 * per lane, non-temporal loads and stores).  *gbs_out receives the better (bytes read + bytes written) /
 * time in GB/s.  Each launch reads and writes exactly `bytes`, so `stream_copy_kernel` is also the kernel
 * of known traffic against which a profiler's HBM byte counters are scaled.  dst and src are device
 * pointers, 16-byte aligned, bytes a multiple of 16 (IL_E_SHAPE otherwise); they may not overlap.
 */
int il_measure_copy_peak(void *dst, const void *src, size_t bytes, int32_t reps, void *stream, double *gbs_out);

#ifdef __cplusplus
}
#endif
#endif /* INTERLOCK_TEST_H */
