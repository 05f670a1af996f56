// Sign-encode kernels (section 3.1 of the paper: value -1 <-> bit 0, +1 <-> bit 1).
//
// All three kernels are pure streaming: 4 bytes read and 1/8 byte written per
// element, so they are bound by HBM bandwidth.  Layout decisions:
//   * row-major matrices: lanes run along K, one v_cmp per 64 elements yields the
//     64-bit word directly (the wave-wide compare mask IS the packed word);
//     a wave covers 16 consecutive words so that 16 independent 256-byte loads are
//     in flight per wave and the 16 words leave in one contiguous 128-byte store.
//   * NCHW images: the packing axis (channel) is strided by H*W floats, so lanes
//     run along pixels (coalesced 256-byte loads per channel) and every lane
//     shift-ORs its own words over a channel loop, then stores its ceil(C/64)
//     words contiguously (packed NHWC).
#include "common.h"

namespace bnn {

// The binarization predicate: +0.0 and -0.0 -> 1, negative and NaN -> 0.
__device__ __forceinline__ bool sign_bit(float v) { return v >= 0.0f; }

constexpr int ENC_WORDS_PER_WAVE = 16;
constexpr int ENC_BLOCK = 256;

__global__ __launch_bounds__(ENC_BLOCK) void encode_rows_kernel(const float *__restrict__ src,
                                                                 int64_t rows, int64_t K,
                                                                 int64_t src_ld, uint64_t *__restrict__ dst,
                                                                 int64_t dst_ld, int64_t Kw,
                                                                 int64_t total_words) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t g0 = ((int64_t)blockIdx.x * (ENC_BLOCK / 64) + wave) * ENC_WORDS_PER_WAVE;
  if (g0 >= total_words) return;
  int64_t row = g0 / Kw;
  int64_t w = g0 - row * Kw;

  // Issue all 16 loads back to back, unconditionally: a lane that has nothing to read
  // (past K in the last word of a row, or past the last row) re-reads element 0 and is
  // masked out afterwards.  Conditional loads would each wait for the previous one.
  float v[ENC_WORDS_PER_WAVE];
  uint32_t okbits = 0;
  int64_t r = row, ww = w;
#pragma unroll
  for (int u = 0; u < ENC_WORDS_PER_WAVE; ++u) {
    const int64_t k = ww * 64 + lane;
    const bool ok = (g0 + u < total_words) && (k < K);
    okbits |= (uint32_t)ok << u;
    v[u] = src[ok ? r * src_ld + k : 0];
    if (++ww == Kw) {
      ww = 0;
      ++r;
    }
  }
  uint64_t mine = 0;
#pragma unroll
  for (int u = 0; u < ENC_WORDS_PER_WAVE; ++u) {
    const uint64_t m = __ballot(((okbits >> u) & 1u) && sign_bit(v[u]));
    if (lane == u) mine = m;
  }
  const int64_t g = g0 + lane;
  if (lane < ENC_WORDS_PER_WAVE && g < total_words) {
    const int64_t rr = g / Kw;
    dst[rr * dst_ld + (g - rr * Kw)] = mine;
  }
}

// Filter bank [D,C,kH,kW] -> packed [D, kH*kW*Cw] in (kh, kw, c) order.  Tiny data
// (a few hundred KB at most), one wave per output word.
__global__ __launch_bounds__(256) void pack_conv_weight_kernel(const float *__restrict__ w, int D, int C,
                                                               int taps, int Cw,
                                                               uint64_t *__restrict__ out,
                                                               int64_t total_words) {
  const int lane = threadIdx.x & 63;
  const int64_t g = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (g >= total_words) return;
  const int cw = (int)(g % Cw);
  const int tap = (int)((g / Cw) % taps);
  const int64_t d = g / ((int64_t)Cw * taps);
  const int c = cw * 64 + lane;
  float v = -1.0f;
  if (c < C) v = w[(d * C + c) * taps + tap];
  const uint64_t m = __ballot(sign_bit(v));
  if (lane == 0) out[g] = m;
}

// NCHW fp32 -> packed pixels [N*OHp*OWp, Cw].  Output pixel (n, oh, ow) samples input
// pixel (oh*sH, ow*sW); with sH = sW = 1 and OHp = H, OWp = W this is the packed NHWC
// image, with the strides of a 1x1 / pad-0 convolution it is the patch matrix itself.
template <int CW>
__global__ __launch_bounds__(256) void encode_nchw_kernel(const float *__restrict__ x, int C, int H, int W,
                                                          int OHp, int OWp, int sH, int sW,
                                                          FastDiv divOW, FastDiv divOH,
                                                          uint64_t *__restrict__ out, uint32_t total_pix,
                                                          int cw_runtime) {
  const uint32_t p = blockIdx.x * 256u + threadIdx.x;
  if (p >= total_pix) return;
  const uint32_t t = fdiv(p, divOW);
  const uint32_t ow = p - t * OWp;
  const uint32_t n = fdiv(t, divOH);
  const uint32_t oh = t - n * OHp;
  const size_t plane = (size_t)H * W;
  const float *px = x + (size_t)n * C * plane + (size_t)(oh * sH) * W + (size_t)ow * sW;
  const int Cw = CW > 0 ? CW : cw_runtime;
  uint64_t *o = out + (size_t)p * Cw;
  uint64_t words[CW > 0 ? CW : 1];
#pragma unroll 1
  for (int cw = 0; cw < Cw; ++cw) {
    const int cbase = cw * 64;
    uint32_t lo = 0, hi = 0;
    if (cbase + 64 <= C) {
      // full word: two groups of 32 channels, loads batched 16 at a time
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        uint32_t acc = 0;
#pragma unroll
        for (int c0 = 0; c0 < 32; c0 += 16) {
          float v[16];
#pragma unroll
          for (int j = 0; j < 16; ++j) v[j] = px[(size_t)(cbase + half * 32 + c0 + j) * plane];
#pragma unroll
          for (int j = 0; j < 16; ++j) acc |= (uint32_t)sign_bit(v[j]) << (c0 + j);
        }
        if (half == 0) lo = acc; else hi = acc;
      }
    } else {
      for (int c = cbase; c < C; ++c) {
        const uint32_t b = (uint32_t)sign_bit(px[(size_t)c * plane]);
        const int bit = c - cbase;
        if (bit < 32) lo |= b << bit; else hi |= b << (bit - 32);
      }
    }
    const uint64_t word = ((uint64_t)hi << 32) | lo;
    if (CW > 0) {
      // static indexing only (cw is a loop counter of an un-unrolled loop)
#pragma unroll
      for (int j = 0; j < (CW > 0 ? CW : 1); ++j)
        if (j == cw) words[j] = word;
    } else {
      o[cw] = word;
    }
  }
  if (CW == 1) {
    o[0] = words[0];
  } else if (CW > 1) {
    // CW is even here: 16-byte stores, contiguous across lanes
    uint4 *o4 = reinterpret_cast<uint4 *>(o);
#pragma unroll
    for (int j = 0; j < (CW > 0 ? CW : 2) / 2; ++j) {
      uint4 q;
      q.x = (uint32_t)words[2 * j];
      q.y = (uint32_t)(words[2 * j] >> 32);
      q.z = (uint32_t)words[2 * j + 1];
      q.w = (uint32_t)(words[2 * j + 1] >> 32);
      o4[j] = q;
    }
  }
}

}  // namespace bnn

using namespace bnn;

extern "C" bnn_status bnn_encode(const float *src, int64_t rows, int64_t K, int64_t src_ld, uint64_t *dst,
                                 int64_t dst_ld, void *stream) {
  if (rows < 0) return BNN_ERR_SHAPE;
  if (K <= 0) return BNN_ERR_SHAPE;
  const int64_t Kw = bnn_packed_words(K);
  if (src_ld < K || dst_ld < Kw) return BNN_ERR_STRIDE;
  if (rows == 0) return BNN_OK;
  if (!src || !dst) return BNN_ERR_NULL;
  if (!aligned16(src) || !aligned16(dst)) return BNN_ERR_ALIGN;
  if (rows > (INT64_MAX / 4) / src_ld) return BNN_ERR_UNSUPPORTED;
  const int64_t total = rows * Kw;
  const int64_t per_block = (int64_t)(ENC_BLOCK / 64) * ENC_WORDS_PER_WAVE;
  const int64_t blocks = (total + per_block - 1) / per_block;
  if (blocks > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  {
    ProfScope ps(KID_ENCODE_ROWS, s);
    hipLaunchKernelGGL(encode_rows_kernel, dim3((unsigned)blocks), dim3(ENC_BLOCK), 0, s, src, rows, K, src_ld,
                       dst, dst_ld, Kw, total);
  }
  return launch_status();
}

extern "C" bnn_status bnn_pack_conv_weight(const float *w, int D, int C, int kH, int kW, uint64_t *w_packed,
                                           void *stream) {
  if (D < 0 || C <= 0 || kH <= 0 || kW <= 0) return BNN_ERR_SHAPE;
  if (D == 0) return BNN_OK;
  if (!w || !w_packed) return BNN_ERR_NULL;
  if (!aligned16(w) || !aligned16(w_packed)) return BNN_ERR_ALIGN;
  const int64_t taps = (int64_t)kH * kW;
  const int64_t Cw = bnn_packed_words(C);
  if (taps > 0x7fff || (int64_t)D * C * taps > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  const int64_t total = (int64_t)D * taps * Cw;
  const int64_t blocks = (total + 3) / 4;
  if (blocks > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  {
    ProfScope ps(KID_PACK_CONV_WEIGHT, s);
    hipLaunchKernelGGL(pack_conv_weight_kernel, dim3((unsigned)blocks), dim3(256), 0, s, w, D, C, (int)taps,
                       (int)Cw, w_packed, total);
  }
  return launch_status();
}

namespace bnn {
// Host launcher used by the im2col / conv drivers.  Arguments are validated by the caller.
bnn_status launch_encode_nchw(const float *x, int N, int C, int H, int W, int OHp, int OWp, int sH, int sW,
                              uint64_t *out, hipStream_t s) {
  const int64_t total = (int64_t)N * OHp * OWp;
  if (total == 0) return BNN_OK;
  if (total > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  const int Cw = (int)bnn_packed_words(C);
  const unsigned blocks = (unsigned)((total + 255) / 256);
  FastDiv dOW((uint32_t)OWp), dOH((uint32_t)OHp);
  ProfScope ps(KID_ENCODE_NCHW, s);
#define BNN_LAUNCH_ENC(CWT)                                                                              \
  hipLaunchKernelGGL(encode_nchw_kernel<CWT>, dim3(blocks), dim3(256), 0, s, x, C, H, W, OHp, OWp, sH, sW, \
                     dOW, dOH, out, (uint32_t)total, Cw)
  switch (Cw) {
    case 1: BNN_LAUNCH_ENC(1); break;
    case 2: BNN_LAUNCH_ENC(2); break;
    case 4: BNN_LAUNCH_ENC(4); break;
    case 8: BNN_LAUNCH_ENC(8); break;
    default: BNN_LAUNCH_ENC(0); break;
  }
#undef BNN_LAUNCH_ENC
  return launch_status();
}
}  // namespace bnn
