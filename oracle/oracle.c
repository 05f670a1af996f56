/*
 * CPU oracle for the binarized convolution / GEMM path.  TEST INFRASTRUCTURE:
 * only the tests, the smoke check and the benchmark's cpu_baseline leg may use
 * it; the product never calls it.
 *
 * Everything here is the plain definition on binary VALUES (-1 / +1 as floats):
 * no bit packing, no popcount, no tiling.  The method of the paper (section 3.2)
 * reaches exactly these results with xnor + bitcount on encodings, so the
 * definition is the oracle.
 *
 * Pins (tests/test_oracle_*.py): the truth table of Table 1, hand-worked 2x2 / 3x3
 * examples, brute force over all sign patterns for tiny K, the identity
 * dot(+-1) = K - 2*hamming with Python big-int popcounts, the per-word formula of
 * section 3.2, torch's CPU conv2d / matmul on +-1 tensors, exact rational
 * arithmetic for the epilogue.
 * The fp32 glue (oracle_conv2d_f32_seq, oracle_fc_f32_seq) fixes a summation
 * order the paper does not give; that convention is pinned by hand-worked cases
 * in which another order, a separately rounded product or skipped padding taps
 * give a different number, and the indexing by small-integer inputs (exact in
 * any order) against torch's float64 convolution / matmul.
 *
 * Build: gcc -O3 -march=x86-64-v3 -ffp-contract=off -fopenmp -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Deterministic binarization Sign(x) (section 4.2) with the encoding rule of
 * section 3.1 (+1 <-> bit 1, -1 <-> bit 0).  The predicate is x >= 0:
 * +0.0 and -0.0 give +1, NaN gives -1. */
static inline float sgn(float v) { return v >= 0.0f ? 1.0f : -1.0f; }

float oracle_sign(float v) { return sgn(v); }

void oracle_sign_array(const float *x, int64_t n, float *s) {
  for (int64_t i = 0; i < n; ++i) s[i] = sgn(x[i]);
}

/* Gemm-Accumulation (section 3.2, first equation) on the binary values of two
 * K-contiguous operands: C[m,n] = sum_k s(A[m,k]) * s(B[n,k]).
 * Every partial sum is an integer of magnitude <= K < 2^24, so the float
 * accumulation is exact. */
void oracle_gemm_pm1(const float *A, const float *B, int64_t M, int64_t N, int64_t K, int32_t *C) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m) {
    for (int64_t n = 0; n < N; ++n) {
      float acc = 0.0f;
      for (int64_t k = 0; k < K; ++k) acc += sgn(A[m * K + k]) * sgn(B[n * K + k]);
      C[m * N + n] = (int32_t)acc;
    }
  }
}

/* One output of the direct convolution (section 2.1, the basic convolution
 * equation) on binary values.  The fp32 input is zero-padded BEFORE the sign,
 * so a tap outside the image has value sign(0) = +1. */
static float conv_point(const float *x, const float *w, int64_t C, int64_t H, int64_t W, int64_t kH,
                        int64_t kW, int64_t sH, int64_t sW, int64_t pH, int64_t pW, int64_t n,
                        int64_t d, int64_t oh, int64_t ow) {
  float acc = 0.0f;
  for (int64_t c = 0; c < C; ++c)
    for (int64_t kh = 0; kh < kH; ++kh)
      for (int64_t kw = 0; kw < kW; ++kw) {
        int64_t ih = oh * sH + kh - pH, iw = ow * sW + kw - pW;
        float xv = 0.0f;
        if (ih >= 0 && ih < H && iw >= 0 && iw < W) xv = x[((n * C + c) * H + ih) * W + iw];
        acc += sgn(w[((d * C + c) * kH + kh) * kW + kw]) * sgn(xv);
      }
  return acc;
}

void oracle_conv2d_pm1(const float *x, const float *w, int64_t N, int64_t C, int64_t H, int64_t W,
                       int64_t D, int64_t kH, int64_t kW, int64_t sH, int64_t sW, int64_t pH,
                       int64_t pW, int32_t *out) {
  int64_t OH = (H + 2 * pH - kH) / sH + 1, OW = (W + 2 * pW - kW) / sW + 1;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t n = 0; n < N; ++n)
    for (int64_t d = 0; d < D; ++d)
      for (int64_t oh = 0; oh < OH; ++oh)
        for (int64_t ow = 0; ow < OW; ++ow)
          out[((n * D + d) * OH + oh) * OW + ow] =
              (int32_t)conv_point(x, w, C, H, W, kH, kW, sH, sW, pH, pW, n, d, oh, ow);
}

/* The same definition evaluated only at the listed flat NCHW output indices. */
void oracle_conv2d_pm1_at(const float *x, const float *w, int64_t N, int64_t C, int64_t H, int64_t W,
                          int64_t D, int64_t kH, int64_t kW, int64_t sH, int64_t sW, int64_t pH,
                          int64_t pW, const int64_t *idx, int64_t n_idx, int32_t *out) {
  int64_t OH = (H + 2 * pH - kH) / sH + 1, OW = (W + 2 * pW - kW) / sW + 1;
  (void)N;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n_idx; ++i) {
    int64_t f = idx[i];
    int64_t ow = f % OW, oh = (f / OW) % OH, d = (f / (OW * OH)) % D, n = f / (OW * OH * D);
    out[i] = (int32_t)conv_point(x, w, C, H, W, kH, kW, sH, sW, pH, pW, n, d, oh, ow);
  }
}

/* Bias step of the forward graph (section 2.2) widened to a per-channel affine
 * map with a single rounding: y = fma(scale[ch], (float)acc, bias[ch]).
 * axis 1: ch = row index; axis 2: ch = column index.  For NCHW conv outputs call
 * with rows = N*D, cols = OH*OW and ch_mod = D (ch = row % D). */
void oracle_scale_bias(const int32_t *acc, int64_t rows, int64_t cols, const float *scale,
                       const float *bias, int axis, int64_t ch_mod, float *y) {
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < cols; ++c) {
      int64_t ch = axis == 1 ? (ch_mod > 0 ? r % ch_mod : r) : c;
      y[r * cols + c] = fmaf(scale[ch], (float)acc[r * cols + c], bias[ch]);
    }
}

/* 2x2 / stride-2 max-pool on int32 planes ([planes, H, W] -> [planes, H/2, W/2]). */
void oracle_maxpool2x2_i32(const int32_t *in, int64_t planes, int64_t H, int64_t W, int32_t *out) {
  int64_t OH = H / 2, OW = W / 2;
  for (int64_t p = 0; p < planes; ++p)
    for (int64_t oh = 0; oh < OH; ++oh)
      for (int64_t ow = 0; ow < OW; ++ow) {
        const int32_t *b = in + (p * H + 2 * oh) * W + 2 * ow;
        int32_t m = b[0];
        if (b[1] > m) m = b[1];
        if (b[W] > m) m = b[W];
        if (b[W + 1] > m) m = b[W + 1];
        out[(p * OH + oh) * OW + ow] = m;
      }
}

/* fp32 convolution with a fixed sequential summation order (c, then kh, then kw),
 * one fma per tap, zero padding contributing fma(0, w, acc) = acc; then the
 * affine map y = fma(scale[d], acc, bias[d]) when scale is given.  Used for the
 * real-valued first layer of the stack. */
void oracle_conv2d_f32_seq(const float *x, const float *w, int64_t N, int64_t C, int64_t H,
                           int64_t W, int64_t D, int64_t kH, int64_t kW, int64_t sH, int64_t sW,
                           int64_t pH, int64_t pW, const float *scale, const float *bias,
                           float *out) {
  int64_t OH = (H + 2 * pH - kH) / sH + 1, OW = (W + 2 * pW - kW) / sW + 1;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t n = 0; n < N; ++n)
    for (int64_t d = 0; d < D; ++d)
      for (int64_t oh = 0; oh < OH; ++oh)
        for (int64_t ow = 0; ow < OW; ++ow) {
          float acc = 0.0f;
          for (int64_t c = 0; c < C; ++c)
            for (int64_t kh = 0; kh < kH; ++kh)
              for (int64_t kw = 0; kw < kW; ++kw) {
                int64_t ih = oh * sH + kh - pH, iw = ow * sW + kw - pW;
                float xv = 0.0f;
                if (ih >= 0 && ih < H && iw >= 0 && iw < W) xv = x[((n * C + c) * H + ih) * W + iw];
                acc = fmaf(xv, w[((d * C + c) * kH + kh) * kW + kw], acc);
              }
          if (scale) acc = fmaf(scale[d], acc, bias[d]);
          out[((n * D + d) * OH + oh) * OW + ow] = acc;
        }
}

/* fp32 fully-connected layer, sequential order over k: acc = fma(x_k, w_k, acc),
 * then + bias.  With sign_input != 0 the input is binarized first (x_k replaced
 * by its binary value), which is how the last real-valued layer of the stack
 * consumes the previous binarized layer. */
void oracle_fc_f32_seq(const float *x, const float *w, const float *bias, int64_t M, int64_t K,
                       int64_t N, int sign_input, float *out) {
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      float acc = 0.0f;
      for (int64_t k = 0; k < K; ++k) {
        float xv = x[m * K + k];
        if (sign_input) xv = sgn(xv);
        acc = fmaf(xv, w[n * K + k], acc);
      }
      if (bias) acc = acc + bias[n];
      out[m * N + n] = acc;
    }
}

/* Threads the parallel loops above actually use (for the benchmark's report). */
int oracle_num_threads(void) {
  int n = 1;
#ifdef _OPENMP
#pragma omp parallel
  {
#pragma omp master
    n = omp_get_num_threads();
  }
#endif
  return n;
}
