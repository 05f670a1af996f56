// Glue kernels of the binarized VGG-small stack and the measurement yardsticks.
// The paper's kernel covers the convolution only (section 4.4); these are the minimal
// correctness-first pieces around it.  The fp32 layers use one thread per output and a
// fixed sequential fma order so that their rounding is reproducible bit for bit (a
// differently rounded value could flip a sign that the next binarized layer consumes).
#include "common.h"
#include "bnn_testing.h"
#include "gemm_rows.inc"

namespace bnn {

__global__ __launch_bounds__(256) void maxpool2x2_kernel(const int32_t *__restrict__ in, int D, int H, int W,
                                                         int32_t *__restrict__ out_i32, float *__restrict__ out_f32,
                                                         const float *__restrict__ scale,
                                                         const float *__restrict__ bias, FastDiv divOW, FastDiv divOH,
                                                         FastDiv divD, uint32_t total) {
  const uint32_t o = blockIdx.x * 256u + threadIdx.x;
  if (o >= total) return;
  const uint32_t OW = W / 2, OH = H / 2;
  const uint32_t t = fdiv(o, divOW);
  const uint32_t ow = o - t * OW;
  const uint32_t plane = fdiv(t, divOH);
  const uint32_t oh = t - plane * OH;
  const int2 r0 = *reinterpret_cast<const int2 *>(in + ((size_t)plane * H + 2 * oh) * W + 2 * ow);
  const int2 r1 = *reinterpret_cast<const int2 *>(in + ((size_t)plane * H + 2 * oh + 1) * W + 2 * ow);
  const int m = max(max(r0.x, r0.y), max(r1.x, r1.y));
  if (out_i32) out_i32[o] = m;
  if (out_f32) {
    const uint32_t d = plane - fdiv(plane, divD) * D;
    out_f32[o] = fmaf(scale[d], (float)m, bias[d]);
  }
}

// One thread per output pixel, all D output channels in groups of CONV_DB accumulators.
// Every output still sees its taps in the order (c, kh, kw), one fma each.  Within a
// group the input value is loaded once and the weights are wave-uniform (scalar loads).
constexpr int CONV_DB = 16;
__global__ __launch_bounds__(256) void conv2d_f32_kernel(const float *__restrict__ x, const float *__restrict__ w,
                                                         int C, int H, int W, int D, int kH, int kW, int sH, int sW,
                                                         int pH, int pW, int OH, int OW,
                                                         const float *__restrict__ scale,
                                                         const float *__restrict__ bias, float *__restrict__ out,
                                                         FastDiv divOW, FastDiv divOH, uint32_t total_pix) {
  const uint32_t p = blockIdx.x * 256u + threadIdx.x;
  if (p >= total_pix) return;
  const uint32_t t = fdiv(p, divOW);
  const uint32_t ow = p - t * OW;
  const uint32_t n = fdiv(t, divOH);
  const uint32_t oh = t - n * OH;
  const int ih0 = (int)(oh * sH) - pH, iw0 = (int)(ow * sW) - pW;
  const float *xn = x + (size_t)n * C * H * W;
  const size_t opix = (size_t)oh * OW + ow;
  const int taps = kH * kW;
  for (int d0 = 0; d0 < D; d0 += CONV_DB) {
    float acc[CONV_DB];
#pragma unroll
    for (int j = 0; j < CONV_DB; ++j) acc[j] = 0.0f;
    for (int c = 0; c < C; ++c)
      for (int kh = 0; kh < kH; ++kh)
        for (int kw = 0; kw < kW; ++kw) {
          const int ih = ih0 + kh, iw = iw0 + kw;
          const bool inside = ih >= 0 && ih < H && iw >= 0 && iw < W;
          const float xv = inside ? xn[((size_t)c * H + ih) * W + iw] : 0.0f;
          const float *wp = w + ((size_t)d0 * C + c) * taps + kh * kW + kw;
#pragma unroll
          for (int j = 0; j < CONV_DB; ++j) {
            const int dj = d0 + j < D ? j : 0;  // clamp: the extra lanes of a ragged group are not stored
            acc[j] = fmaf(xv, wp[(size_t)dj * C * taps], acc[j]);
          }
        }
#pragma unroll
    for (int j = 0; j < CONV_DB; ++j) {
      const int d = d0 + j;
      if (d < D) {
        float r = acc[j];
        if (scale) r = fmaf(scale[d], r, bias[d]);
        out[((size_t)n * D + d) * OH * OW + opix] = r;
      }
    }
  }
}

// One workgroup per (ROWS rows of x, 16 outputs).  The whole K extent (up to FC_KC) of those
// rows of x and w is staged in LDS by all 256 threads with every global load in flight at once,
// so memory latency is paid once; then thread (output j, row r) runs the sequential fma chain
// over k, which is the floor for this layer (the summation order over k is ascending as
// specified, so a chain cannot be split).  Longer rows take several passes over the two LDS
// tiles.  The chains read both operands from LDS (32 bytes per 4 steps and thread), so LDS
// bandwidth, not the chain, bounds a workgroup: ROWS = 4 (one computing wave, the other three
// only stage) spreads a small layer over four times as many compute units as ROWS = 16.
constexpr int FC_NB = 16;
constexpr int FC_KC = 1024;
constexpr int FC_RS = FC_KC + 4;  // row stride in floats: 16-byte reads of different rows spread over the banks
template <int ROWS>
__global__ __launch_bounds__(256) void fc_f32_kernel(const float *__restrict__ x, const float *__restrict__ w,
                                                     const float *__restrict__ bias, int64_t M, int64_t K, int64_t N,
                                                     int sign_input, float *__restrict__ out, int n_groups) {
  __shared__ __attribute__((aligned(16))) float sx[ROWS * FC_RS];
  __shared__ __attribute__((aligned(16))) float sw[FC_NB * FC_RS];
  const int64_t m0 = (int64_t)(blockIdx.x / n_groups) * ROWS;
  const int64_t n0 = (int64_t)(blockIdx.x % n_groups) * FC_NB;
  const int tid = threadIdx.x;
  const int r = tid % ROWS, j = tid / ROWS;
  const bool computes = tid < ROWS * FC_NB;  // whole waves: ROWS * 16 is a multiple of 64
  const bool vec = (K & 3) == 0;  // rows start 16-byte aligned (the bases are)
  float acc = 0.0f;
  for (int64_t k0 = 0; k0 < K; k0 += FC_KC) {
    const int kc = (int)((K - k0) < FC_KC ? (K - k0) : FC_KC);
    if (vec) {
      constexpr int Q = FC_KC / 4;                    // 16-byte pieces per row
      constexpr int PER = (ROWS + FC_NB) * Q / 256;   // pieces per thread: rows of x first, then rows of w
      float4 v[PER];
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        const int idx = i * 256 + tid;
        const int rr = idx / Q, kk = (idx % Q) * 4;
        v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (kk < kc) {
          if (rr < ROWS) {
            if (m0 + rr < M) v[i] = *reinterpret_cast<const float4 *>(x + (m0 + rr) * K + k0 + kk);
          } else if (n0 + (rr - ROWS) < N) {
            v[i] = *reinterpret_cast<const float4 *>(w + (n0 + (rr - ROWS)) * K + k0 + kk);
          }
        }
      }
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        const int idx = i * 256 + tid;
        const int rr = idx / Q, kk = (idx % Q) * 4;
        float4 t = v[i];
        if (rr < ROWS) {
          if (sign_input) {
            t.x = t.x >= 0.0f ? 1.0f : -1.0f; t.y = t.y >= 0.0f ? 1.0f : -1.0f;
            t.z = t.z >= 0.0f ? 1.0f : -1.0f; t.w = t.w >= 0.0f ? 1.0f : -1.0f;
          }
          *reinterpret_cast<float4 *>(&sx[rr * FC_RS + kk]) = t;
        } else {
          *reinterpret_cast<float4 *>(&sw[(rr - ROWS) * FC_RS + kk]) = t;
        }
      }
    } else {
      for (int idx = tid; idx < (ROWS + FC_NB) * FC_KC; idx += 256) {
        const int rr = idx / FC_KC, kk = idx % FC_KC;
        float t = 0.0f;
        if (kk < kc) {
          if (rr < ROWS) {
            if (m0 + rr < M) t = x[(m0 + rr) * K + k0 + kk];
            if (sign_input) t = t >= 0.0f ? 1.0f : -1.0f;
          } else if (n0 + (rr - ROWS) < N) {
            t = w[(n0 + (rr - ROWS)) * K + k0 + kk];
          }
        }
        if (rr < ROWS) sx[rr * FC_RS + kk] = t;
        else sw[(rr - ROWS) * FC_RS + kk] = t;
      }
    }
    __syncthreads();
    if (computes) {
      const float *px = &sx[r * FC_RS], *pw = &sw[j * FC_RS];
      int kk = 0;
      // 32 k per round; the sixteen 16-byte LDS reads of the next round are issued before the
      // chain of the current one, so their latency hides behind its 32 dependent fma
      if (kc >= 32) {
        float4 a[8], b[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          a[u] = *reinterpret_cast<const float4 *>(px + 4 * u);
          b[u] = *reinterpret_cast<const float4 *>(pw + 4 * u);
        }
        for (; kk + 32 <= kc; kk += 32) {
          float4 an[8], bn[8];
          const int nx = kk + 64 <= kc ? kk + 32 : kk;  // last round: re-read this one (unused)
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            an[u] = *reinterpret_cast<const float4 *>(px + nx + 4 * u);
            bn[u] = *reinterpret_cast<const float4 *>(pw + nx + 4 * u);
          }
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            acc = fmaf(a[u].x, b[u].x, acc);
            acc = fmaf(a[u].y, b[u].y, acc);
            acc = fmaf(a[u].z, b[u].z, acc);
            acc = fmaf(a[u].w, b[u].w, acc);
          }
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            a[u] = an[u];
            b[u] = bn[u];
          }
        }
      }
      for (; kk + 4 <= kc; kk += 4) {
        const float4 a = *reinterpret_cast<const float4 *>(px + kk);
        const float4 b = *reinterpret_cast<const float4 *>(pw + kk);
        acc = fmaf(a.x, b.x, acc);
        acc = fmaf(a.y, b.y, acc);
        acc = fmaf(a.z, b.z, acc);
        acc = fmaf(a.w, b.w, acc);
      }
      for (; kk < kc; ++kk) acc = fmaf(px[kk], pw[kk], acc);
    }
    __syncthreads();
  }
  if (computes && m0 + r < M && n0 + j < N) {
    if (bias) acc = acc + bias[n0 + j];
    out[(m0 + r) * N + n0 + j] = acc;
  }
}

// Yardstick 0: 64 independent xor + popcount-accumulate pairs per round from registers and
// nothing else in the loop body but eight cheap updates of the xor operands (so nothing can be
// hoisted); the compiler schedules the xors freely.
__global__ __launch_bounds__(256) void valu_probe_kernel(int32_t *__restrict__ sink, int iters) {
  const uint32_t tid = blockIdx.x * 256u + threadIdx.x;
  uint32_t a[8], b[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    b[j] = tid * 2654435761u + j * 40503u;
    a[j] = 0x9e3779b9u * (j + 1) ^ tid;
  }
  int acc[64];
#pragma unroll
  for (int i = 0; i < 64; ++i) acc[i] = 0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 64; ++i) {
      const uint32_t x = a[i >> 3] ^ b[i & 7];
      asm volatile("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc[i]) : "v"(x));
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) a[j] += b[j];
  }
  int tot = 0;
#pragma unroll
  for (int i = 0; i < 64; ++i) tot += acc[i];
  sink[tid] = tot;
}

// Yardstick 1: the GEMM's own per-row statements (8 rows x TN columns x 8 dwords, xor operand
// in a scalar register, one-cycle yield after each pair) run from registers with no loads at
// all: the issue ceiling of exactly the instruction sequence the GEMM loop consists of.
template <int TN>
__global__ __launch_bounds__(256) void valu_rows_probe_kernel(int32_t *__restrict__ sink, int iters, uint32_t seed) {
  const uint32_t tid = blockIdx.x * 256u + threadIdx.x;
  typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));
  u32x8 a[8], b[TN];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int d = 0; d < 8; ++d) a[i][d] = seed * (uint32_t)(i * 8 + d + 1) + 0x9e3779b9u;
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int d = 0; d < 8; ++d) b[j][d] = tid * 2654435761u + (uint32_t)(j * 8 + d) * 40503u;
  int acc[8][TN];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = 0;
  for (int it = 0; it < iters; ++it) {
    uint32_t t0, t1;
#define BNN_BV(j, d) b[j][d]
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if constexpr (TN == 4) BNN_GEMM_ROW_4(acc[i], a[i], BNN_BV, t0, t1);
      else BNN_GEMM_ROW_2(acc[i], a[i], BNN_BV, t0, t1);
    }
#undef BNN_BV
#pragma unroll
    for (int j = 0; j < TN; ++j) b[j][0] += 1u;
  }
  int tot = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) tot += acc[i][j];
  sink[tid] = tot;
}

__global__ __launch_bounds__(256) void copy_probe_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                                         size_t n16) {
  size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
#pragma unroll
  for (int u = 0; u < 4; ++u, i += 256)
    if (i < n16) dst[i] = src[i];
}

}  // namespace bnn

using namespace bnn;

extern "C" bnn_status bnn_maxpool2x2(const int32_t *in, int N, int D, int H, int W, int32_t *out_i32, float *out_f32,
                                     const float *scale, const float *bias, void *stream) {
  if (N < 0 || D < 0 || H <= 0 || W <= 0 || (H & 1) || (W & 1)) return BNN_ERR_SHAPE;
  if (N == 0 || D == 0) return BNN_OK;
  if (!in || (!out_i32 && !out_f32)) return BNN_ERR_NULL;
  if (out_f32 && (!scale || !bias)) return BNN_ERR_NULL;
  if (!aligned16(in) || (out_i32 && !aligned16(out_i32)) || (out_f32 && !aligned16(out_f32))) return BNN_ERR_ALIGN;
  const int64_t total = (int64_t)N * D * (H / 2) * (W / 2);
  if (total > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  {
    ProfScope ps(KID_MAXPOOL, s);
    hipLaunchKernelGGL(maxpool2x2_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, in, D, H, W, out_i32,
                       out_f32, scale, bias, FastDiv((uint32_t)(W / 2)), FastDiv((uint32_t)(H / 2)),
                       FastDiv((uint32_t)D), (uint32_t)total);
  }
  return launch_status();
}

extern "C" bnn_status bnn_conv2d_f32(const float *x, const float *w, int N, int C, int H, int W, int D, int kH, int kW,
                                     int sH, int sW, int pH, int pW, const float *scale, const float *bias, float *out,
                                     void *stream) {
  bnn_status st = check_conv_geometry(N, C, H, W, kH, kW, sH, sW, pH, pW);
  if (st != BNN_OK) return st;
  if (D < 0) return BNN_ERR_SHAPE;
  if (N == 0 || D == 0) return BNN_OK;
  if (!x || !w || !out) return BNN_ERR_NULL;
  if ((scale == nullptr) != (bias == nullptr)) return BNN_ERR_NULL;
  if (!aligned16(x) || !aligned16(w) || !aligned16(out)) return BNN_ERR_ALIGN;
  const int64_t OH = bnn_conv_out_dim(H, kH, sH, pH), OW = bnn_conv_out_dim(W, kW, sW, pW);
  const int64_t total = (int64_t)N * OH * OW;
  if (total > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  if (C == 3 && kH == 3 && kW == 3) {
    // the network's first layer: the matrix-core chains shared with bnn_conv2d_f32_sign
    ProfScope ps(KID_CONV_F32, s);
    return launch_conv2d_f32_k27(x, w, N, H, W, D, sH, sW, pH, pW, scale, bias, out, s);
  }
  {
    ProfScope ps(KID_CONV_F32, s);
    hipLaunchKernelGGL(conv2d_f32_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, x, w, C, H, W, D, kH,
                       kW, sH, sW, pH, pW, (int)OH, (int)OW, scale, bias, out, FastDiv((uint32_t)OW),
                       FastDiv((uint32_t)OH), (uint32_t)total);
  }
  return launch_status();
}

extern "C" bnn_status bnn_fc_f32(const float *x, const float *w, const float *bias, int64_t M, int64_t K, int64_t N,
                                 int sign_input, float *out, void *stream) {
  if (M < 0 || N < 0 || K <= 0) return BNN_ERR_SHAPE;
  if (M == 0 || N == 0) return BNN_OK;
  if (!x || !w || !out) return BNN_ERR_NULL;
  if (!aligned16(x) || !aligned16(w) || !aligned16(out)) return BNN_ERR_ALIGN;
  const int64_t n_groups = (N + FC_NB - 1) / FC_NB;
  // 16 rows per workgroup when that already gives every compute unit one; else 4
  const bool small = ((M + 15) / 16) * n_groups < 256;
  const int64_t m_groups = small ? (M + 3) / 4 : (M + 15) / 16;
  if (m_groups * n_groups > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  {
    ProfScope ps(KID_FC_F32, s);
    const dim3 grid((unsigned)(m_groups * n_groups)), block(256);
    if (small)
      hipLaunchKernelGGL(fc_f32_kernel<4>, grid, block, 0, s, x, w, bias, M, K, N, sign_input, out, (int)n_groups);
    else
      hipLaunchKernelGGL(fc_f32_kernel<16>, grid, block, 0, s, x, w, bias, M, K, N, sign_input, out, (int)n_groups);
  }
  return launch_status();
}

extern "C" bnn_status bnn_valu_peak_probe(int32_t *sink, int blocks, int iters, int kind, void *stream) {
  if (blocks < 0 || iters < 0 || (kind != 0 && kind != 2 && kind != 4)) return BNN_ERR_SHAPE;
  if (blocks == 0) return BNN_OK;
  if (!sink) return BNN_ERR_NULL;
  if (!aligned16(sink)) return BNN_ERR_ALIGN;
  hipStream_t s = (hipStream_t)stream;
  {
    ProfScope ps(KID_VALU_PROBE, s);
    const dim3 g((unsigned)blocks), b(256);
    // a round of the row statements is 8 x TN x 8 pairs: iters is scaled so that every kind
    // issues 2 * 64 * iters lane-operations per lane
    if (kind == 2) hipLaunchKernelGGL(valu_rows_probe_kernel<2>, g, b, 0, s, sink, iters / 2, 1u);
    else if (kind == 4) hipLaunchKernelGGL(valu_rows_probe_kernel<4>, g, b, 0, s, sink, iters / 4, 1u);
    else hipLaunchKernelGGL(valu_probe_kernel, g, b, 0, s, sink, iters);
  }
  return launch_status();
}

extern "C" bnn_status bnn_copy_probe(const void *src, void *dst, size_t n_bytes, void *stream) {
  if (n_bytes % 16) return BNN_ERR_SHAPE;
  if (n_bytes == 0) return BNN_OK;
  if (!src || !dst) return BNN_ERR_NULL;
  if (!aligned16(src) || !aligned16(dst)) return BNN_ERR_ALIGN;
  const size_t n16 = n_bytes / 16;
  const size_t blocks = (n16 + 1023) / 1024;
  if (blocks > 0x7fffffffULL) return BNN_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  {
    ProfScope ps(KID_COPY_PROBE, s);
    hipLaunchKernelGGL(copy_probe_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (const uint4 *)src, (uint4 *)dst,
                       n16);
  }
  return launch_status();
}
