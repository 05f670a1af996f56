/*
 * bnn_testing.h -- entry points for tests and measurements; NOT part of the library's ABI and
 * not meant for applications.  The *_testing_* calls are the calls of bnn.h with the kernel
 * variant chosen by the caller instead of by the size heuristic; every variant computes the
 * values bnn.h specifies, and nothing set here outlives the call.  Only the kernel-timing hook
 * (bnn_prof_*) keeps state between calls: a list of HIP events, which never changes what a
 * call computes or launches.
 */
#ifndef BNN_TESTING_H_
#define BNN_TESTING_H_

#include "bnn.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Tile configurations of the Xnor-Bitcount GEMM (section 3.2), argument `cfg` below:
 *   -1  the size heuristic (what bnn.h's entry points use)
 *    1  32 x 256 tile      2  32 x 64       3  64 x 256      4  32 x 128      6  64 x 128
 *    7  one wave per 8 x 64 tile, operand B read straight from memory (small problems)
 *    8  one wave per 8 x 128 tile, likewise
 *    9  as 7 with the reduction axis split over the four waves of a workgroup
 *   13 .. 18  long rows, few outputs: one wave per (8 * T) x 64 tile slice, B kept in registers
 *       across the T row groups, the reduction axis split over the S waves of a workgroup:
 *       (T, S) = (4, 4), (4, 8), (2, 8), (2, 4), (4, 2), (2, 2)
 *   19, 20  the latency form of the implicit-GEMM convolution (32 x 64 tiles, one column per lane,
 *       the reduction axis split over 4 / 2 slices inside a workgroup); needs an even number of
 *       words per pixel
 *   10  the short-row kernel (rows of two or four words, four consecutive columns per lane,
 *       16-byte stores), 8 rows per wave;   11, 12  the same with 16 / 32 rows per wave
 * A value that a call cannot use (the packed epilogue needs a 32- or 64-row tile with two or
 * four column groups; 7 to 18 exist for an explicit B with int32 / fp32 output only, 10 to 12
 * only where N, the leading dimensions and the pixels per image are multiples of 4) selects the
 * heuristic for that call.
 * `lean`: 1 = convolutions whose geometry allows it gather their patches with the table-driven
 * loader (what bnn.h's entry points do); 0 = always the general loader.
 */

/* bnn_xnor_gemm_epilogue (and, with Y == NULL, bnn_xnor_gemm) on tile configuration cfg. */
BNN_API bnn_status bnn_testing_xnor_gemm_epilogue(const uint64_t *A, int64_t lda, const uint64_t *B, int64_t ldb,
                                                  int64_t M, int64_t N, int64_t K, int32_t *C, int64_t ldc, float *Y,
                                                  int64_t ldy, const float *scale, const float *bias,
                                                  bnn_ch_axis axis, int cfg, void *stream);

/* bnn_conv2d on tile configuration cfg and gather `lean`. */
BNN_API bnn_status bnn_testing_conv2d(const float *x, const uint64_t *w_packed, int N, int C, int H, int W, int D,
                                      int kH, int kW, int sH, int sW, int pH, int pW, int32_t *out_i32,
                                      float *out_f32, const float *scale, const float *bias, void *workspace,
                                      size_t workspace_bytes, int cfg, int lean, void *stream);

/* bnn_conv2d_packed on tile configuration cfg and gather `lean`. */
BNN_API bnn_status bnn_testing_conv2d_packed(const uint64_t *x_packed, const uint64_t *w_packed, int N, int C, int H,
                                             int W, int D, int kH, int kW, int sH, int sW, int pH, int pW, int pool,
                                             int32_t *out_i32, float *out_f32, uint64_t *out_packed,
                                             const float *scale, const float *bias, int cfg, int lean,
                                             void *stream);

/*
 * bnn_xnor_gemm_mfma_fp4_expanded on a chosen workgroup tile (rows x columns of C):
 *   -1 the choice of bnn.h's entry point;  0 128 x 128;  1 256 x 128;  2 128 x 256.
 * Other values: BNN_ERR_SHAPE.
 */
BNN_API bnn_status bnn_testing_xnor_gemm_mfma_fp4_expanded(const uint8_t *A4, int64_t lda_bytes, const uint8_t *B4,
                                                           int64_t ldb_bytes, int32_t *C, int64_t ldc, int64_t M,
                                                           int64_t N, int64_t K, int tile, void *stream);

/* ---- measurement helpers ------------------------------------------------------------ */

/*
 * Kernel timing.  While enabled, every kernel the library launches is bracketed by a
 * pair of HIP events recorded on the caller's stream (host objects, created on first
 * use and kept until bnn_prof_enable(0)).  At most BNN_PROF_MAX_RECORDS launches are
 * recorded between two resets; later ones run untimed.  Not thread-safe.
 */
#define BNN_PROF_MAX_RECORDS 4096
BNN_API bnn_status bnn_prof_enable(int enable);
BNN_API bnn_status bnn_prof_reset(void);
BNN_API int64_t bnn_prof_count(void);
/* Synchronises on record i's end event, then returns its kernel id and duration. */
BNN_API bnn_status bnn_prof_get(int64_t i, int *kernel_id, float *milliseconds);
BNN_API const char *bnn_kernel_name(int kernel_id);

/*
 * bnn_valu_peak_probe -- a microbenchmark, not part of the method: every lane issues
 * 2 * 64 * iters vector lane-operations (xor + popcount-accumulate pairs) from registers,
 * no loads; the grid is `blocks` workgroups of 256 threads.  sink [blocks*256] int32
 * receives a value that depends on all of them.
 *   kind 0  independent pairs, both operands in vector registers, scheduled by the compiler
 *   kind 2 / 4  the GEMM's own row statements for 2 / 4 column groups per lane (xor operand
 *           in a scalar register, each xor directly followed by its popcount, one-cycle
 *           yield after each pair); iters should be a multiple of kind
 * Other kinds: BNN_ERR_SHAPE.
 */
BNN_API bnn_status bnn_valu_peak_probe(int32_t *sink, int blocks, int iters, int kind, void *stream);

/*
 * bnn_copy_probe -- plain device copy of n_bytes (multiple of 16) used as the yardstick
 * for achievable HBM bandwidth and for scaling hardware byte counters.
 */
BNN_API bnn_status bnn_copy_probe(const void *src, void *dst, size_t n_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* BNN_TESTING_H_ */
