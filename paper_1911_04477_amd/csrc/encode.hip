// Sign-encode kernels (section 3.1 of the paper: value -1 <-> bit 0, +1 <-> bit 1).
//
// All three kernels are pure streaming: 4 bytes read and 1/8 byte written per
// element, so they are bound by HBM bandwidth.  Layout decisions:
//   * row-major matrices: lanes run along K, one v_cmp per 64 elements yields the
//     64-bit word directly (the wave-wide compare mask IS the packed word);
//     a wave covers 16 consecutive words so that 16 independent 256-byte loads are
//     in flight per wave and the 16 words leave in one contiguous 128-byte store.
//     The fp32 input is read exactly once, with non-temporal loads (5.44 -> 5.76 TB/s).
//   * NCHW images: the packing axis (channel) is strided by H*W floats, so lanes
//     run along pixels (coalesced 256-byte loads per channel) and every lane
//     shift-ORs 32 channels at a time; the four waves of a workgroup share the
//     channel axis of 64 pixels and assemble the packed NHWC words through LDS.
#include "common.h"

namespace bnn {

// The binarization predicate: +0.0 and -0.0 -> 1, negative and NaN -> 0.
__device__ __forceinline__ bool sign_bit(float v) { return v >= 0.0f; }

constexpr int ENC_BLOCK = 256;

constexpr int ENC_WORDS_PER_WAVE = 16;
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
    v[u] = __builtin_nontemporal_load(&src[ok ? r * src_ld + k : 0]);  // read once: keep it out of the caches
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
//
// A workgroup owns 64 consecutive output pixels (one per lane).  The channel axis is cut
// into granules of 32 channels (one half word) dealt round-robin to the workgroup's four
// waves, so four times as many waves stream as there are pixel groups and each lane has
// 32 independent plane-strided loads in flight per granule.  The half words meet in LDS
// and leave as one contiguous run of 64 * Cw words.  (A variant with four pixels per lane
// and 16-byte loads measured no faster, from cache or from HBM, and was dropped.)
constexpr int ENCN_PIX = 64;
__global__ __launch_bounds__(256) void encode_nchw_kernel(const float *__restrict__ x, int C, int H, int W,
                                                          int OHp, int OWp, int sH, int sW, FastDiv divOW,
                                                          FastDiv divOH, uint64_t *__restrict__ out,
                                                          uint32_t total_pix, int Cw) {
  extern __shared__ uint32_t s_half[];  // [64 pixels][2*Cw + 1]
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t p0 = blockIdx.x * (uint32_t)ENCN_PIX;
  const uint32_t p = p0 + lane;
  const uint32_t pc = p < total_pix ? p : total_pix - 1;  // lanes past the end re-read the last pixel
  const uint32_t t = fdiv(pc, divOW);
  const uint32_t ow = pc - t * OWp;
  const uint32_t n = fdiv(t, divOH);
  const uint32_t oh = t - n * OHp;
  const size_t plane = (size_t)H * W;
  // Address = wave-uniform 64-bit base (first image of the workgroup, channel plane) + a
  // 32-bit per-lane byte offset: one VGPR of address per lane instead of one pair per load.
  // The host checks that the offset (the images a workgroup can span) fits.
  const uint32_t n0 = fdiv(fdiv(p0 < total_pix ? p0 : total_pix - 1, divOW), divOH);
  const uint32_t off =
      (uint32_t)(((size_t)(n - n0) * C * plane + (size_t)(oh * sH) * W + (size_t)ow * sW) * sizeof(float));
  const char *xb = reinterpret_cast<const char *>(x + (size_t)n0 * C * plane);
#define BNN_ENC_LD(c) \
  __builtin_nontemporal_load(reinterpret_cast<const float *>(xb + (size_t)(c) * plane * sizeof(float) + off))
  const int G = 2 * Cw;  // granules, the last ones possibly partial or empty
  const int rs = G + 1;
  for (int g = wave; g < G; g += 4) {
    const int c0 = g * 32;
    const int left = C - c0;  // real channels in this granule
    uint32_t acc = 0;
    if (left >= 32) {
      float v[32];
#pragma unroll
      for (int j = 0; j < 32; ++j) v[j] = BNN_ENC_LD(c0 + j);
#pragma unroll
      for (int j = 0; j < 32; ++j) acc |= (uint32_t)sign_bit(v[j]) << j;
    } else if (left > 0) {
      // channels past C re-read the last channel and are masked out
      float v[32];
#pragma unroll
      for (int j = 0; j < 32; ++j) v[j] = BNN_ENC_LD(c0 + (j < left ? j : left - 1));
#pragma unroll
      for (int j = 0; j < 32; ++j) acc |= (uint32_t)sign_bit(v[j]) << j;
      acc &= (1u << left) - 1u;
    }
    s_half[lane * rs + g] = acc;
  }
#undef BNN_ENC_LD
  __syncthreads();
  // 64 * Cw words, contiguous in global memory from pixel p0
  const uint32_t nwords = (uint32_t)ENCN_PIX * (uint32_t)Cw;
  const uint64_t limit = (uint64_t)total_pix * (uint64_t)Cw;
  uint64_t *o = out + (size_t)p0 * Cw;
  for (uint32_t j = threadIdx.x; j < nwords; j += 256u) {
    if ((uint64_t)p0 * Cw + j >= limit) break;
    const uint32_t pix = j / (uint32_t)Cw, cw = j - pix * (uint32_t)Cw;
    const uint32_t lo = s_half[pix * rs + 2 * cw], hi = s_half[pix * rs + 2 * cw + 1];
    o[j] = ((uint64_t)hi << 32) | lo;
  }
}

// The same encode for a column stride above 1 (the sampled pixels of a strided 1x1 / pad-0
// convolution).  A wave's load then uses only every sW-th float of the sectors it touches, rows
// between the sampled ones are skipped, and what bounds the kernel is how many independent
// requests are in flight rather than bytes: a read-only kernel over the same addresses tops out
// at 60 % of the streaming rate.  So every wave works alone on 64 pixels x ONE granule of 16
// channels (16 loads in flight per lane), keeps its 16 sign bits per pixel and writes them
// straight to its quarter of the pixel's word: no LDS, no barrier, four times as many waves.
// The partial-word stores meet in the L2; the packed output is 1/32 of the input.  (Measured on
// the 64 x 200 x 56 x 56 input with stride 2: 19.4 us against 24.1 us for the kernel above;
// for stride 1 the kernel above is the faster one at every size tried.)
constexpr int ENCS_GR = 16;
__global__ __launch_bounds__(256) void encode_nchw_sampled_kernel(const float *__restrict__ x, int C, int H, int W,
                                                                  int OHp, int OWp, int sH, int sW, FastDiv divOW,
                                                                  FastDiv divOH, uint16_t *__restrict__ out,
                                                                  uint32_t total_pix, int Cw) {
  const uint32_t p = blockIdx.x * 256u + threadIdx.x;
  const int g = blockIdx.y;  // granule: channels [16 g, 16 g + 16)
  const uint32_t pc = p < total_pix ? p : total_pix - 1;  // lanes past the end re-read the last pixel
  const uint32_t t = fdiv(pc, divOW);
  const uint32_t ow = pc - t * OWp;
  const uint32_t n = fdiv(t, divOH);
  const uint32_t oh = t - n * OHp;
  const size_t plane = (size_t)H * W;
  const float *xp = x + (size_t)n * C * plane + (size_t)(oh * sH) * W + (size_t)ow * sW;
  const int c0 = g * ENCS_GR;
  const int left = C - c0;  // real channels in this granule; <= 0 for the padding granules of the last word
  uint32_t acc = 0;
  if (left > 0) {
    float v[ENCS_GR];
#pragma unroll
    for (int j = 0; j < ENCS_GR; ++j)  // channels past C re-read the last channel and are masked out
      v[j] = __builtin_nontemporal_load(xp + (size_t)(c0 + (j < left ? j : left - 1)) * plane);
#pragma unroll
    for (int j = 0; j < ENCS_GR; ++j) acc |= (uint32_t)sign_bit(v[j]) << j;
    if (left < ENCS_GR) acc &= (1u << left) - 1u;
  }
  if (p < total_pix) out[(size_t)p * (4 * Cw) + g] = (uint16_t)acc;
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
  const unsigned blocks = (unsigned)((total + ENCN_PIX - 1) / ENCN_PIX);
  const size_t lds = (size_t)ENCN_PIX * (2 * Cw + 1) * sizeof(uint32_t);
  if (lds > 64 * 1024) return BNN_ERR_UNSUPPORTED;  // C > 8128 channels
  // 32-bit per-lane byte offsets: a workgroup's 64 pixels span at most `span` images past its first
  const int64_t span = (ENCN_PIX + (int64_t)OHp * OWp - 1) / ((int64_t)OHp * OWp);
  if ((span + 1) * (int64_t)C * H * W * 4 > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  FastDiv dOW((uint32_t)OWp), dOH((uint32_t)OHp);
  ProfScope ps(KID_ENCODE_NCHW, s);
  if (sW > 1 && 4 * Cw <= 65535) {
    const dim3 grid((unsigned)((total + 255) / 256), (unsigned)(4 * Cw));
    hipLaunchKernelGGL(encode_nchw_sampled_kernel, grid, dim3(256), 0, s, x, C, H, W, OHp, OWp, sH, sW, dOW, dOH,
                       reinterpret_cast<uint16_t *>(out), (uint32_t)total, Cw);
    return launch_status();
  }
  hipLaunchKernelGGL(encode_nchw_kernel, dim3(blocks), dim3(256), lds, s, x, C, H, W, OHp, OWp, sH, sW, dOW, dOH, out,
                     (uint32_t)total, Cw);
  return launch_status();
}
}  // namespace bnn
