/*
 * bnn.h -- C ABI of the MI355X (gfx950) binarized convolution / GEMM library.
 *
 * The library implements the forward path of a binarized convolutional layer as
 * described in "A Computing Kernel for Network Binarization on PyTorch"
 * (arXiv 1911.04477): tensors are sign-encoded into 1-bit words (section 3.1),
 * the input is im2col-lowered (section 2.1) and the Gemm-Accumulation is replaced
 * by Xnor-Bitcount (section 3.2).
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - Pointers named in the argument lists are DEVICE pointers unless stated
 *    otherwise.  The caller owns every buffer; the library allocates and frees no
 *    device memory and never synchronises: work is enqueued on `stream`
 *    (a hipStream_t passed as void*; NULL = the default stream).
 *  - Base pointers must be 16-byte aligned (BNN_ERR_ALIGN otherwise).
 *  - All argument checks happen on the host before any launch; on error nothing
 *    is launched.  A failed launch is reported as BNN_ERR_HIP.
 *  - Empty problems (a zero row / column / batch count) return BNN_OK without a
 *    launch.  A reduction length K <= 0 is BNN_ERR_SHAPE.
 *  - What a call computes and which kernels it launches depend on its arguments and the
 *    device only: the library keeps no settings between calls.
 *
 * Packed format (part of the ABI; section 3.1: value -1 <-> bit 0, +1 <-> bit 1)
 * -----------------------------------------------------------------------------
 *  A packed row of K binary values is ceil(K/64) uint64 words.  Element k lives in
 *  bit (k mod 64), least-significant bit first, of word (k div 64).  Bits past K in
 *  the last word are 0.  On a little-endian machine the same bytes viewed as
 *  uint32 are the paper's uint32_t packing with 32 values per word.
 *  Binarization is Sign(x) (section 4.2) with the predicate x >= 0:  +0.0 and -0.0
 *  encode as 1, negative values and NaN as 0.
 *
 * Packed convolution operands
 * ---------------------------
 *  The reduction axis of a convolution is ordered (kh, kw, c) with c innermost, and
 *  every tap (kh, kw) owns ceil(C/64) whole words (pad bits 0 in BOTH operands), so
 *  a packed patch / filter row has bnn_conv_kwords(C,kH,kW) = kH*kW*ceil(C/64)
 *  words.  Because the exclusive-or of two pad bits is 0 they do not contribute,
 *  and the result uses the true K = C*kH*kW.
 *
 * Implemented range (BNN_ERR_UNSUPPORTED beyond it; nothing is launched)
 * ----------------------------------------------------------------------
 *  Every limit is checked on the host.  They follow from 32-bit indices inside the kernels:
 *   - GEMM entry points: M, K below 2^31, N at most 2^31 - 257; operand A at most 4 GiB (M * lda * 8 bytes).
 *     The MFMA ablations: K below 2^29 (int8), below 2^24 (both fp4 forms).
 *   - Convolutions: N*H*W below 2^31 pixels; N*C*H*W at most 2^33 values; N*OH*OW at most
 *     2^29 output pixels; N*OH*OW*bnn_conv_kwords() below 2^31 words; kH*kW at most 32767;
 *     the packed filter bank at most 4 GiB; D*N*OH*OW at most 2^34 outputs; the packed
 *     reduction below 2^31 bits.  Entry points that take an fp32 image additionally need
 *     C <= 8128 and two consecutive images within 2 GiB (C*H*W*4 bytes each).
 *   - bnn_encode: rows * ceil(K/64) below 2^37 words.
 *   - bnn_conv2d_f32_sign: C*kH*kW at most 32.  bnn_control_conv2d_f32: C*kH*kW below 2^24.
 *   - The glue kernels (pool, real-valued convolution, fully-connected layer): fewer than
 *     2^31 output elements.
 */
#ifndef BNN_H_
#define BNN_H_

#include <stddef.h>
#include <stdint.h>

/* The library is built with hidden default visibility; only what is declared here (and the
 * test / measurement entry points of bnn_testing.h) is exported. */
#define BNN_API __attribute__((visibility("default")))

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  BNN_OK = 0,
  BNN_ERR_NULL = 1,        /* a required pointer is NULL */
  BNN_ERR_SHAPE = 2,       /* a dimension is negative, K <= 0, or an output dimension is < 1 */
  BNN_ERR_STRIDE = 3,      /* a leading dimension is smaller than the row it must hold */
  BNN_ERR_ALIGN = 4,       /* a base pointer is not 16-byte aligned */
  BNN_ERR_WORKSPACE = 5,   /* workspace_bytes is smaller than the matching *_workspace_bytes() */
  BNN_ERR_HIP = 6,         /* the HIP runtime reported an error at launch */
  BNN_ERR_UNSUPPORTED = 7  /* valid request outside the implemented range (sizes over 2^31 elements per operand, ...) */
} bnn_status;

typedef enum { BNN_CH_NONE = 0, BNN_CH_ROW = 1, BNN_CH_COL = 2 } bnn_ch_axis;

/* Human-readable name of a status code (static storage, never NULL). */
BNN_API const char *bnn_status_str(bnn_status s);

/* ceil(K/64): uint64 words per packed row of K values; 0 for K <= 0. */
BNN_API int64_t bnn_packed_words(int64_t K);

/* kH*kW*ceil(C/64): words per packed patch / filter row; 0 for non-positive input. */
BNN_API int64_t bnn_conv_kwords(int C, int kH, int kW);

/* floor((in + 2*pad - k)/stride) + 1, or 0 when that is not positive / arguments invalid. */
BNN_API int64_t bnn_conv_out_dim(int64_t in, int64_t k, int64_t stride, int64_t pad);

/*
 * bnn_encode -- sign-encode a row-major fp32 matrix along its rows (section 3.1: the
 * packing runs along the rows, i.e. along the reduction axis; the paper packs 32 values
 * per uint32_t, this library 64 per uint64_t).
 *   src     [rows, K] fp32, row stride src_ld floats (src_ld >= K)
 *   dst     [rows, ceil(K/64)] uint64, row stride dst_ld words (dst_ld >= ceil(K/64));
 *           pad bits of the last word are written as 0; words between ceil(K/64)
 *           and dst_ld are not touched.
 */
BNN_API bnn_status bnn_encode(const float *src, int64_t rows, int64_t K, int64_t src_ld, uint64_t *dst,
                      int64_t dst_ld, void *stream);

/*
 * bnn_pack_conv_weight -- encode a filter bank (section 3.1: the weight skips im2col
 * and is stored pre-encoded as a [D, K^2 C / wordsize] bit matrix).
 *   w         [D, C, kH, kW] fp32 contiguous
 *   w_packed  [D, bnn_conv_kwords(C,kH,kW)] uint64 contiguous, (kh, kw, c) order.
 */
BNN_API bnn_status bnn_pack_conv_weight(const float *w, int D, int C, int kH, int kW, uint64_t *w_packed,
                                void *stream);

/*
 * bnn_im2col_packed -- lower an fp32 NCHW image batch to packed patch rows
 * (section 2.1 im2col, section 3.1 input encoding).  The fp32 input is zero-padded
 * BEFORE binarization, so a tap outside the image encodes as +1 (bit 1) for each of
 * the C real channels.
 *   x     [N, C, H, W] fp32 contiguous
 *   cols  [N*OH*OW, bnn_conv_kwords(C,kH,kW)] uint64 contiguous; row p = (n*OH + oh)*OW + ow
 *   workspace  scratch of at least bnn_im2col_workspace_bytes(...) bytes (may be NULL
 *              when that is 0); contents undefined afterwards.
 */
BNN_API bnn_status bnn_im2col_packed(const float *x, int N, int C, int H, int W, int kH, int kW, int sH,
                             int sW, int pH, int pW, uint64_t *cols, void *workspace,
                             size_t workspace_bytes, void *stream);
BNN_API size_t bnn_im2col_workspace_bytes(int N, int C, int H, int W, int kH, int kW, int sH, int sW,
                                  int pH, int pW);

/*
 * bnn_xnor_gemm -- Xnor-Bitcount GEMM (section 3.2, Table 1) in the exclusive-or
 * form, valid for every K:   C[m,n] = K - 2 * sum_w popcount(A[m,w] XOR B[n,w]).
 * For K a multiple of 32 this equals the paper's sum of 2*Bitcount(xnor) - 32.
 *   A  [M, ceil(K/64)] uint64, row stride lda words;  B  [N, ceil(K/64)], row stride ldb
 *      (both operands K-contiguous).  Bits past K in the last word are ignored
 *      (masked), whatever they hold.
 *   C  [M, N] int32 row-major, row stride ldc elements (ldc >= N).
 */
BNN_API bnn_status bnn_xnor_gemm(const uint64_t *A, int64_t lda, const uint64_t *B, int64_t ldb, int32_t *C,
                         int64_t ldc, int64_t M, int64_t N, int64_t K, void *stream);

/*
 * bnn_xnor_gemm_epilogue -- the same GEMM followed by the per-channel affine map that
 * stands for the bias step of the forward graph (section 2.2):
 *   Y[m,n] = fma(scale[ch], (float)C[m,n], bias[ch])   (one rounding),
 *   ch = m for BNN_CH_ROW, n for BNN_CH_COL.
 *   C (int32, ldc) and Y (fp32, ldy) may each be NULL, not both.  With Y non-NULL,
 *   scale and bias are required (M or N floats according to axis) and axis must not
 *   be BNN_CH_NONE.
 */
BNN_API bnn_status bnn_xnor_gemm_epilogue(const uint64_t *A, int64_t lda, const uint64_t *B, int64_t ldb,
                                  int64_t M, int64_t N, int64_t K, int32_t *C, int64_t ldc, float *Y,
                                  int64_t ldy, const float *scale, const float *bias,
                                  bnn_ch_axis axis, void *stream);

/*
 * bnn_conv2d -- binarized convolution forward (the forward graph of Figure 3):
 * input encode + packed im2col, Xnor-Bitcount GEMM against the pre-encoded filter
 * bank, result written straight into the NCHW output (no col2im pass), optional
 * per-output-channel affine map.
 *   x         [N, C, H, W] fp32 contiguous
 *   w_packed  [D, bnn_conv_kwords(C,kH,kW)] uint64 from bnn_pack_conv_weight
 *   out_i32   [N, D, OH, OW] int32 or NULL;  out_f32 same shape fp32 or NULL (not both NULL)
 *   scale, bias  [D] fp32, required iff out_f32 != NULL:
 *             out_f32 = fma(scale[d], (float)acc, bias[d])
 *   workspace at least bnn_conv2d_workspace_bytes(...) bytes (device, 16-byte aligned): it
 *             receives the packed NHWC image (1 bit per input value) the GEMM gathers its
 *             taps from; no patch matrix is materialised.
 */
BNN_API bnn_status bnn_conv2d(const float *x, const uint64_t *w_packed, int N, int C, int H, int W, int D,
                      int kH, int kW, int sH, int sW, int pH, int pW, int32_t *out_i32,
                      float *out_f32, const float *scale, const float *bias, void *workspace,
                      size_t workspace_bytes, void *stream);
BNN_API size_t bnn_conv2d_workspace_bytes(int N, int C, int H, int W, int kH, int kW, int sH, int sW, int pH,
                                  int pW);

/*
 * bnn_conv2d_noalloc -- bnn_conv2d for callers that cannot allocate device memory and have no
 * workspace to hand over: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments (minus the workspace), same kernels, same results; the packed
 * image goes to a fixed array of BNN_CONV2D_NOALLOC_MAX_BYTES in device memory that the library
 * holds on every GPU it runs on until the process ends.  The call allocates and frees nothing.
 *   - A problem whose bnn_conv2d_workspace_bytes() exceeds the limit returns BNN_ERR_WORKSPACE
 *     (checked first, before any HIP call; nothing is launched).
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 *     streams, two threads) race on it and must be serialised by the caller.  The array keeps the
 *     previous call's contents; every word a call reads it has written first, so nothing needs
 *     clearing.
 *   - The first call on a device looks up the array's device address (once per device, kept for
 *     the life of the process); make that first call outside a stream capture.  BNN_ERR_HIP if
 *     the address cannot be obtained.
 */
#define BNN_CONV2D_NOALLOC_MAX_BYTES (8u << 20)
BNN_API bnn_status bnn_conv2d_noalloc(const float *x, const uint64_t *w_packed, int N, int C, int H, int W,
                                      int D, int kH, int kW, int sH, int sW, int pH, int pW, int32_t *out_i32,
                                      float *out_f32, const float *scale, const float *bias, void *stream);
BNN_API size_t bnn_conv2d_noalloc_max_bytes(void);

/*
 * bnn_conv2d_packed -- the same forward graph with activations kept packed between
 * layers (1 bit per activation in memory): the input is a packed NHWC image, and with the
 * binarizing epilogue the output is the packed NHWC image the next layer consumes.
 *   x_packed  [N, H, W, ceil(C/64)] uint64: pixel-major, channel c in bit (c mod 64) of word
 *             (c div 64), pad bits 0 (what bnn_conv2d_f32_sign or this function writes)
 *   w_packed  [D, bnn_conv_kwords(C,kH,kW)] from bnn_pack_conv_weight
 *   Exactly one kind of output per call:
 *     out_i32 and/or out_f32  [N, D, OH, OW] NCHW as in bnn_conv2d (pool must be 0), or
 *     out_packed [N, OH', OW', ceil(D/64)] uint64 with
 *         bit d = ( fma(scale[d], (float)a, bias[d]) >= 0 ),
 *         a = acc[n,d,oh,ow] for pool == 0 (OH' = OH, OW' = OW), or the maximum of acc over
 *         the 2x2 window for pool == 2 (OH' = OH/2, OW' = OW/2; OH and OW must be even):
 *         conv -> max-pool on int32 -> affine -> sign, the block order of the stack.
 *   scale, bias [D] are required for out_f32 and out_packed.  No workspace is needed: the
 *   patch matrix is never materialised.
 */
BNN_API bnn_status bnn_conv2d_packed(const uint64_t *x_packed, const uint64_t *w_packed, int N, int C, int H,
                             int W, int D, int kH, int kW, int sH, int sW, int pH, int pW, int pool,
                             int32_t *out_i32, float *out_f32, uint64_t *out_packed,
                             const float *scale, const float *bias, void *stream);

/*
 * bnn_conv2d_f32_sign -- real-valued first layer of the stack with binarized output:
 * bnn_conv2d_f32 (same fixed summation order) followed by fma(scale[d], acc, bias[d]) and
 * the sign, written as a packed NHWC image [N, OH, OW, ceil(D/64)].  Limited to
 * C*kH*kW <= 32 taps (BNN_ERR_UNSUPPORTED otherwise).
 */
BNN_API bnn_status bnn_conv2d_f32_sign(const float *x, const float *w, int N, int C, int H, int W, int D,
                               int kH, int kW, int sH, int sW, int pH, int pW, const float *scale,
                               const float *bias, uint64_t *out_packed, void *stream);

/*
 * bnn_pack_fc_weight_nhwc -- encode the weight of a fully-connected layer whose input is a
 * flattened NCHW map [C, H, W] so that it can be multiplied with that map's packed NHWC
 * form: w [Nout, C*H*W] fp32 -> w_packed [Nout, H*W*ceil(C/64)] uint64 with the reduction
 * axis re-ordered to (h, w, c), each pixel padded to whole words.  (A permutation applied to
 * the reduction axis of both operands does not change the product.)
 */
BNN_API bnn_status bnn_pack_fc_weight_nhwc(const float *w, int64_t Nout, int C, int H, int W,
                                   uint64_t *w_packed, void *stream);

/* ---- glue kernels of the binarized VGG-small stack (not part of the paper's kernel,
 *      which covers convolution only -- section 4.4) -------------------------------- */

/*
 * bnn_maxpool2x2 -- 2x2 / stride-2 max-pool on int32 planes, optionally followed by the
 * affine map on the pooled value.
 *   in       [N, D, H, W] int32 (H, W even);  out_i32 / out_f32 [N, D, H/2, W/2], one may be NULL
 *   out_f32 = fma(scale[d], (float)max, bias[d]);  scale, bias [D] required iff out_f32.
 */
BNN_API bnn_status bnn_maxpool2x2(const int32_t *in, int N, int D, int H, int W, int32_t *out_i32,
                          float *out_f32, const float *scale, const float *bias, void *stream);

/*
 * bnn_conv2d_f32 -- real-valued convolution for the first layer of the stack.
 * Summation order is fixed: acc = 0; for c, kh, kw (row-major): acc = fma(x, w, acc)
 * with zero padding; then, when scale != NULL, out = fma(scale[d], acc, bias[d]).
 *   x [N,C,H,W], w [D,C,kH,kW], out [N,D,OH,OW], all fp32 contiguous.
 */
BNN_API bnn_status bnn_conv2d_f32(const float *x, const float *w, int N, int C, int H, int W, int D, int kH,
                          int kW, int sH, int sW, int pH, int pW, const float *scale,
                          const float *bias, float *out, void *stream);

/*
 * bnn_fc_f32 -- real-valued fully-connected layer for the last layer of the stack.
 *   out[m,n] = (acc = 0; for k ascending: acc = fma(xk, w[n,k], acc)) + bias[n]
 *   where xk = x[m,k], or its binary value (x >= 0 ? +1 : -1) when sign_input != 0.
 *   x [M,K], w [N,K], bias [N] or NULL, out [M,N], all fp32 contiguous.
 */
BNN_API bnn_status bnn_fc_f32(const float *x, const float *w, const float *bias, int64_t M, int64_t K,
                      int64_t N, int sign_input, float *out, void *stream);

/* ---- ablation --------------------------------------------------------------------------- */

/*
 * bnn_xnor_gemm_mfma_i8 -- ABLATION of bnn_xnor_gemm, same arguments and bit-identical
 * result, computed on the matrix cores: CDNA4 has no 1-bit MFMA, so every packed bit is
 * expanded on the fly to an int8 (0 / 1) and V_MFMA_I32_32X32X32_I8 counts the positions
 * where both operands are +1; K - 2*popcount(a XOR b) follows from that count and the two
 * rows' own +1 counts.  Measured beside the VALU path, not used by any other entry point.
 */
BNN_API bnn_status bnn_xnor_gemm_mfma_i8(const uint64_t *A, int64_t lda, const uint64_t *B, int64_t ldb,
                                 int32_t *C, int64_t ldc, int64_t M, int64_t N, int64_t K,
                                 void *stream);

/*
 * bnn_xnor_gemm_mfma_fp4 -- the same ABLATION on the 4-bit floating-point matrix instruction
 * (V_MFMA_SCALE_F32_32X32X64_F8F6F4, both operands E2M1): every packed bit becomes the code for
 * 0.0 or 0.5, both operands carry the block scale 2, and the fp32 accumulator counts the
 * positions where both are +1 exactly.  Same arguments, same bit-identical int32 result;
 * K below 2^24 (BNN_ERR_UNSUPPORTED beyond).  Not used by any other entry point.
 */
BNN_API bnn_status bnn_xnor_gemm_mfma_fp4(const uint64_t *A, int64_t lda, const uint64_t *B, int64_t ldb,
                                          int32_t *C, int64_t ldc, int64_t M, int64_t N, int64_t K,
                                          void *stream);

/*
 * bnn_expand_fp4, bnn_xnor_gemm_mfma_fp4_expanded -- third ABLATION: the matrix-core GEMM with the
 * expansion taken out of it.  The two forms above spend most of their time turning bits into
 * matrix operands; here that is a separate streaming pass, and the GEMM reads operands kept in
 * memory at 4 bits per value.
 *   E2M1 row format: value k of a row is the 4-bit floating-point code of +1.0 (0x2) or -1.0
 *   (0xA) in nibble k % 2 (low nibble first) of byte k / 2; the row is padded with the code of
 *   0.0 (0x0) to a multiple of 64 values, bnn_fp4_row_bytes(K) = 32 * ceil(K / 64) bytes.
 * bnn_expand_fp4: src [rows, src_ld] packed sign words (device, read; bits past K ignored),
 *   dst [rows, dst_ld_bytes] bytes (device, written), dst_ld_bytes >= bnn_fp4_row_bytes(K) and a
 *   multiple of 16.  Both 16-byte aligned.
 * bnn_xnor_gemm_mfma_fp4_expanded: A4 [M, lda_bytes], B4 [N, ldb_bytes] in that format (device,
 *   read), C [M, ldc] int32 (device, written) = sum over k of a_k * b_k, the same number as
 *   bnn_xnor_gemm gives on the packed rows (section 3.2), exact in the fp32 accumulator of
 *   V_MFMA_SCALE_F32_32X32X64_F8F6F4 for K below 2^24 (BNN_ERR_UNSUPPORTED beyond).
 * Errors as bnn_xnor_gemm; strides in bytes, multiples of 16.  Not used by any other entry point.
 */
BNN_API int64_t bnn_fp4_row_bytes(int64_t K);
BNN_API bnn_status bnn_expand_fp4(const uint64_t *src, int64_t rows, int64_t K, int64_t src_ld, uint8_t *dst,
                                  int64_t dst_ld_bytes, void *stream);
BNN_API bnn_status bnn_xnor_gemm_mfma_fp4_expanded(const uint8_t *A4, int64_t lda_bytes, const uint8_t *B4,
                                                   int64_t ldb_bytes, int32_t *C, int64_t ldc, int64_t M,
                                                   int64_t N, int64_t K, void *stream);

/*
 * bnn_conv2d_mfma_fp4_expanded -- the same ABLATION as a convolution (sections 2.1 and 3.2): the
 * patches are gathered inside the GEMM from a 4-bit NHWC image, so the patch matrix (kH*kW times
 * the image) never exists.  out[n, d, oh, ow] as bnn_conv2d's int32 output, taps outside the image
 * counting as +1.
 *   x4 [N, H, W, C / 2 bytes]: bnn_expand_fp4 of the packed NHWC image taken as N*H*W rows of C
 *     values; w4 [D, kH*kW*C / 2 bytes]: bnn_expand_fp4 of bnn_pack_conv_weight's rows
 *     (K = kH*kW*C); out_i32 [N, D, OH, OW] (device, written).  All 16-byte aligned.
 *   C must be a multiple of 64 (BNN_ERR_UNSUPPORTED otherwise), C*kH*kW below 2^24.
 * Errors as bnn_conv2d.  Not used by any other entry point.
 */
BNN_API bnn_status bnn_conv2d_mfma_fp4_expanded(const uint8_t *x4, const uint8_t *w4, int N, int C, int H, int W,
                                                int D, int kH, int kW, int sH, int sW, int pH, int pW,
                                                int32_t *out_i32, void *stream);

/* ---- control group --------------------------------------------------------------------- */

/*
 * bnn_control_conv2d_f32 -- the paper's fp32 "control group" (section 4.4): the same
 * binarized convolution computed as an ordinary real-valued GEMM, for restating the kernel's
 * speed-up on this machine.  out[n, d, oh, ow] = sum over (c, kh, kw) of sign(w) * sign(x),
 * taps outside the image counting as sign(0) = +1; every value is an exact integer in fp32
 * and equals bnn_conv2d's int32 result.  Implicit GEMM on the fp32 matrix cores, no workspace.
 *   x   [N, C, H, W] fp32 (device), w [D, C, kH, kW] fp32 (device), out [N, D, OH, OW] fp32
 *   (device, written).  All three 16-byte aligned.  C*kH*kW < 2^24.
 * Errors as bnn_conv2d.  Not used by any other entry point.
 */
BNN_API bnn_status bnn_control_conv2d_f32(const float *x, const float *w, int N, int C, int H, int W,
                                  int D, int kH, int kW, int sH, int sW, int pH, int pW,
                                  float *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* BNN_H_ */
