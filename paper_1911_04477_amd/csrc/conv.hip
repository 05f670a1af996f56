// Binarized convolution drivers: the forward graph of Figure 3 of the paper (encode the
// input, pre-encoded weight, Xnor-Bitcount, reshape to the output feature map).
//  * The reshape (col2im of section 2.1) costs nothing: the GEMM store writes each
//    accumulator straight to its NCHW position.
//  * The patch matrix of im2col is never materialised: the GEMM gathers its B tiles from
//    the packed NHWC image (implicit GEMM).
//  * bnn_conv2d_packed keeps activations packed between layers: packed NHWC in, and with
//    the binarizing epilogue packed NHWC out (2x2 max-pool, affine map and sign fused into
//    the GEMM store), so a stack of binarized layers moves 1 bit per activation.
//  * bnn_conv2d_f32_sign is the real-valued first layer producing that packed format.
#include <mutex>

#include "common.h"
#include "bnn_testing.h"

namespace bnn {

bnn_status launch_encode_nchw(const float *x, int N, int C, int H, int W, int OHp, int OWp, int sH, int sW,
                              uint64_t *out, hipStream_t s);

static void fill_geom(ConvGeom &g, const uint64_t *act, int N, int C, int H, int W, int kH, int kW, int sH, int sW, int pH,
                      int pW, int pool) {
  g.act = act;
  g.Nimg = N; g.C = C; g.H = H; g.W = W;
  g.Cw = (int)bnn_packed_words(C);
  g.OH = (int)bnn_conv_out_dim(H, kH, sH, pH);
  g.OW = (int)bnn_conv_out_dim(W, kW, sW, pW);
  g.kH = kH; g.kW = kW; g.sH = sH; g.sW = sW; g.pH = pH; g.pW = pW;
  g.pool = pool;
  g.divCw = FastDiv((uint32_t)g.Cw);
  g.divKW = FastDiv((uint32_t)kW);
  g.divOW = FastDiv((uint32_t)(pool ? g.OW / 2 : g.OW));
  g.divOH = FastDiv((uint32_t)(pool ? g.OH / 2 : g.OH));
}

// GEMM over an already packed NHWC image; arguments validated by the callers.
static bnn_status conv_from_packed(const uint64_t *act, const uint64_t *w_packed, int N, int C, int H, int W, int D,
                                   int kH, int kW, int sH, int sW, int pH, int pW, int pool, int32_t *out_i32,
                                   float *out_f32, uint64_t *out_packed, const float *scale, const float *bias,
                                   hipStream_t s, const GemmTune &tune) {
  const int64_t OH = bnn_conv_out_dim(H, kH, sH, pH), OW = bnn_conv_out_dim(W, kW, sW, pW);
  const int64_t Kw = bnn_conv_kwords(C, kH, kW);
  const int64_t cols = pool ? 4 * ((int64_t)N * (OH / 2) * (OW / 2)) : (int64_t)N * OH * OW;
  GemmParams p = {};
  p.A = reinterpret_cast<const uint32_t *>(w_packed);
  p.B = nullptr;
  p.lda32 = 2 * Kw;
  p.ldb = Kw;
  p.M = D;
  p.N = (int)cols;
  p.Kbits = (int)(Kw * 64);  // pad bits are 0 in both operands: they cancel in the exclusive-or
  p.Kformula = C * kH * kW;
  p.Kd = (int)(Kw * 2);
  p.Kw64 = (int)Kw;
  p.b_vec16 = 0;
  p.C = out_i32;
  p.Y = out_f32;
  p.ldc = p.ldy = OH * OW;
  p.scale = scale;
  p.bias = bias;
  p.axis = BNN_CH_ROW;
  p.OHW = (uint32_t)(OH * OW);
  p.divOHW = FastDiv((uint32_t)(OH * OW));
  p.img_stride = (int64_t)D * OH * OW;
  fill_geom(p.g, act, N, C, H, W, kH, kW, sH, sW, pH, pW, pool);
  p.outp = out_packed;
  p.cw_out = (int)bnn_packed_words(D);
  return run_gemm(p, 1, out_packed ? 1 : 0, s, tune);
}

static bnn_status conv_limits(int N, int C, int H, int W, int D, int kH, int kW, int sH, int sW, int pH, int pW) {
  const int64_t OH = bnn_conv_out_dim(H, kH, sH, pH), OW = bnn_conv_out_dim(W, kW, sW, pW);
  const int64_t P = (int64_t)N * OH * OW;
  const int64_t Kw = bnn_conv_kwords(C, kH, kW);
  // column count, 32-bit byte offsets into the filter bank, output elements, pixels, and the
  // reduction length in bits (an int in the kernel's parameters)
  if (P > 0x7ffffff0LL / 4 || (int64_t)D * 8 * Kw > 0xffffffffLL || (int64_t)D * P > 0x7fffffffLL * 8 ||
      (int64_t)N * H * W > 0x7fffffffLL || Kw * 64 > 0x7fffffffLL)
    return BNN_ERR_UNSUPPORTED;
  return BNN_OK;
}

// ---- real-valued first layer with binarized, packed output ----------------------------------
// One thread per output pixel.  The input patch (K = C*kH*kW <= 32 taps) sits in registers.
// The filter bank, scale and bias are wave-uniform, so they are read through the constant
// address space with scalar loads and enter v_fma as the scalar operand (an LDS copy would
// make the CU's single LDS pipe the bottleneck: four SIMDs reading 7 x 16 bytes per channel).
// Every output channel is the sequential fma chain over (c, kh, kw), then fma(scale, acc,
// bias); only its sign is kept, 64 channels per stored word.
constexpr int F32S_KMAX = 32;
#define BNN_CONST_AS __attribute__((address_space(4)))
typedef const float BNN_CONST_AS *cf32_ptr;

template <int KT>  // KT = K when known at compile time (27 for 3x3x3), else 0
__global__ __launch_bounds__(256) void conv2d_f32_sign_kernel(const float *__restrict__ x, const float *w_, int C,
                                                              int H, int W, int D, int kH, int kW, int sH, int sW,
                                                              int pH, int pW, int OH, int OW, const float *scale_,
                                                              const float *bias_, uint64_t *__restrict__ outp,
                                                              int cw_out, FastDiv divOW, FastDiv divOH,
                                                              uint32_t total_pix, int K_rt) {
  const int K = KT > 0 ? KT : K_rt;
  const cf32_ptr w = (cf32_ptr)(uintptr_t)w_;
  const cf32_ptr scale = (cf32_ptr)(uintptr_t)scale_;
  const cf32_ptr bias = (cf32_ptr)(uintptr_t)bias_;
  const uint32_t p = blockIdx.x * 256u + threadIdx.x;
  if (p >= total_pix) return;
  const uint32_t t = fdiv(p, divOW);
  const uint32_t ow = p - t * OW;
  const uint32_t n = fdiv(t, divOH);
  const uint32_t oh = t - n * OH;
  const int ih0 = (int)(oh * sH) - pH, iw0 = (int)(ow * sW) - pW;
  const float *xn = x + (size_t)n * C * H * W;
  const int taps = kH * kW;
  constexpr int KU = KT > 0 ? KT : F32S_KMAX;
  float xv[KU];
#pragma unroll
  for (int k = 0; k < KU; ++k) {
    float v = 0.0f;
    if (k < K) {
      const int c = k / taps, r = k - c * taps;
      const int kh = r / kW, kw = r - kh * kW;
      const int ih = ih0 + kh, iw = iw0 + kw;
      if (ih >= 0 && ih < H && iw >= 0 && iw < W) v = xn[((size_t)c * H + ih) * W + iw];
    }
    xv[k] = v;
  }
  for (int d0 = 0; d0 < D; d0 += 64) {
    uint32_t lo = 0, hi = 0;
    const int dn = D - d0 < 64 ? D - d0 : 64;
#pragma unroll 4
    for (int dd = 0; dd < dn; ++dd) {
      const cf32_ptr wr = w + (size_t)(d0 + dd) * K;
      float acc = 0.0f;
#pragma unroll
      for (int k = 0; k < KU; ++k)
        if (k < K) acc = fmaf(xv[k], wr[k], acc);
      const uint32_t bit = fmaf(scale[d0 + dd], acc, bias[d0 + dd]) >= 0.0f ? 1u : 0u;
      if (dd < 32) lo |= bit << dd; else hi |= bit << (dd - 32);
    }
    outp[(size_t)p * cw_out + (d0 >> 6)] = ((uint64_t)hi << 32) | lo;
  }
}

// ---- the 3x3x3 layer (K = 27) on the fp32 matrix cores --------------------------------------
// V_MFMA_F32_32X32X1_2B_F32 multiplies a 32 x 1 column by a 1 x 32 row and adds the 32 x 32
// product to its accumulator, for two independent blocks at once; one reduction step at a time,
// each output element goes through exactly the fused multiply-add chain over (c, kh, kw) that
// the general kernel above runs (checked bit for bit against fmaf chains, denormals, infinities
// and signed zeros included), at twice the rate of unpacked vector multiply-adds.
//   rows (operand A)    : 32 output channels; lanes l and l + 32 hold the same filter tap
//   columns (operand B) : the wave's 64 pixels, block 0 = pixels 0..31, block 1 = pixels 32..63;
//                         lane l supplies the patch value of pixel l
//   accumulators        : register r of block b, lane l = channel 8*(r/4) + 4*(l/32) + r%4 of
//                         pixel 32*b + l%32
// A workgroup stages the filter taps of up to 128 channels in LDS ([tap][channel], odd row
// stride), then each wave walks over its pixel groups: 27 clamped loads per lane, four channel
// groups x 27 matrix instructions, and the affine map + sign on the vector unit.
constexpr int C1M_CH = 128;   // channels per workgroup (blockIdx.y)
constexpr int C1M_RS = 129;   // LDS row stride of the tap-major filter tile
typedef float c1m_v32f __attribute__((ext_vector_type(32)));

__device__ __forceinline__ uint32_t c1m_spread_nibbles(uint32_t m) {
  // nibble q of a 16-bit mask -> bits 8q .. 8q+3
  return (m & 0xFu) | ((m & 0xF0u) << 4) | ((m & 0xF00u) << 8) | ((m & 0xF000u) << 12);
}

// Stage the filter taps of channels ch0 .. ch0 + 127 tap-major in LDS (read [channel][tap]
// contiguously; channels past D are zero) and their scale / bias (past D, or without an affine
// map: fma(0, acc, -1) < 0, so such bits are 0).
__device__ __forceinline__ void c1m_stage_filters(float *sTap, float *sSc, float *sBi, const float *__restrict__ w,
                                                  const float *__restrict__ scale, const float *__restrict__ bias,
                                                  int ch0, int nch, bool affine) {
  const int tid = threadIdx.x;
  for (int idx = tid; idx < 27 * C1M_CH; idx += 256) {
    const int ch = idx / 27, k = idx - 27 * ch;
    sTap[k * C1M_RS + ch] = ch < nch ? w[(size_t)ch0 * 27 + idx] : 0.0f;
  }
  if (tid < C1M_CH) {
    const bool real = tid < nch && affine;
    sSc[tid] = real ? scale[ch0 + tid] : 0.0f;
    sBi[tid] = real ? bias[ch0 + tid] : -1.0f;
  }
}

// Issue the 27 loads of pixel p's patch: every tap unconditionally from a clamped (always
// readable) position; bit r of `inside` says whether tap (r / 3, r % 3) lies in the image.
__device__ __forceinline__ void c1m_issue_patch(const float *__restrict__ x, uint32_t p, uint32_t total_pix, int H,
                                                int W, int sH, int sW, int pH, int pW, int OH, int OW, FastDiv divOW,
                                                FastDiv divOH, float (&raw)[27], uint32_t &inside) {
  const bool pv = p < total_pix;
  const uint32_t pc = pv ? p : 0u;
  const uint32_t t = fdiv(pc, divOW);
  const uint32_t ow = pc - t * OW;
  const uint32_t n = fdiv(t, divOH);
  const uint32_t oh = t - n * OH;
  const int ih0 = (int)(oh * sH) - pH, iw0 = (int)(ow * sW) - pW;
  const float *xn = x + (size_t)n * 3 * H * W;
  uint32_t rok = 0, cok = 0;
  int roff[3], coff[3];
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    const int ih = ih0 + j, iw = iw0 + j;
    rok |= (uint32_t)(pv && ih >= 0 && ih < H) << j;
    cok |= (uint32_t)(iw >= 0 && iw < W) << j;
    roff[j] = (ih < 0 ? 0 : (ih >= H ? H - 1 : ih)) * W;
    coff[j] = iw < 0 ? 0 : (iw >= W ? W - 1 : iw);
  }
  inside = 0;
#pragma unroll
  for (int r = 0; r < 9; ++r) inside |= (((rok >> (r / 3)) & (cok >> (r % 3))) & 1u) << r;
#pragma unroll
  for (int k = 0; k < 27; ++k) {
    const int c = k / 9, r = k % 9;
    raw[k] = xn[(size_t)c * H * W + roff[r / 3] + coff[r % 3]];
  }
}

// 27 dependent matrix instructions: channel group g (32 channels) x this wave's 64 pixels.
__device__ __forceinline__ c1m_v32f c1m_chain(const float *wg, const float (&xv)[27]) {
  c1m_v32f acc;
#pragma unroll
  for (int r = 0; r < 32; ++r) acc[r] = 0.0f;
#pragma unroll
  for (int k = 0; k < 27; ++k) acc = __builtin_amdgcn_mfma_f32_32x32x1f32(wg[k * C1M_RS], xv[k], acc, 0, 0, 0);
  return acc;
}

// Affine map and sign of one channel group's accumulators -> the 32 channel bits of this
// lane's own pixel.  Lanes l and l + 32 hold the two channel halves of a pixel: l < 32 keeps
// its block-0 bits and receives the partner's, l >= 32 likewise with block 1.
__device__ __forceinline__ uint32_t c1m_sign_bits(const c1m_v32f &acc, const float *sSc, const float *sBi, int g,
                                                  int half) {
  // rows descend so that every sign is shifted in with one add-with-carry: m = 2 * m + (y >= 0)
  uint32_t m0 = 0u, m1 = 0u;
#pragma unroll
  for (int q = 3; q >= 0; --q) {
    const float4 sc = *reinterpret_cast<const float4 *>(sSc + 32 * g + 8 * q + 4 * half);
    const float4 bi = *reinterpret_cast<const float4 *>(sBi + 32 * g + 8 * q + 4 * half);
    const float scv[4] = {sc.x, sc.y, sc.z, sc.w}, biv[4] = {bi.x, bi.y, bi.z, bi.w};
#pragma unroll
    for (int e = 3; e >= 0; --e) {
      const int rr = 4 * q + e;
      const float y0 = fmaf(scv[e], acc[rr], biv[e]), y1 = fmaf(scv[e], acc[16 + rr], biv[e]);
      asm("v_cmp_le_f32 vcc, 0, %1\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc" : "+v"(m0) : "v"(y0) : "vcc");
      asm("v_cmp_le_f32 vcc, 0, %1\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc" : "+v"(m1) : "v"(y1) : "vcc");
    }
  }
  const uint32_t own = half ? m1 : m0;
  const uint32_t got = (uint32_t)__shfl_xor((int)(half ? m0 : m1), 32);
  const uint32_t lo = half ? got : own, hi = half ? own : got;  // channels 8q+0..3 / 8q+4..7
  return c1m_spread_nibbles(lo) | (c1m_spread_nibbles(hi) << 4);
}

// Packed-sign output.
// On this chip the fp32 matrix instructions and the vector ALU do not run side by side (vector
// instructions placed between the matrix instructions of a chain lengthen it by their full
// issue time, measured), so nothing is gained by interleaving the sign step with the next chain:
// the loop is the plain sequence loads, one chain per group of 32 channels followed by its sign
// step, store, and several resident waves per SIMD cover the load latency.
__global__ __launch_bounds__(256, 4) void conv2d_f32_k27_mfma_sign_kernel(
    const float *__restrict__ x, const float *__restrict__ w, int H, int W, int D, int sH, int sW, int pH, int pW,
    int OH, int OW, const float *__restrict__ scale, const float *__restrict__ bias, uint64_t *__restrict__ outp,
    int cw_out, FastDiv divOW, FastDiv divOH, uint32_t total_pix, uint32_t ngroups, int groups_per_wave) {
  __shared__ float sTap[27 * C1M_RS];
  __shared__ __attribute__((aligned(16))) float sSc[C1M_CH];
  __shared__ __attribute__((aligned(16))) float sBi[C1M_CH];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int half = lane >> 5, l32 = lane & 31;
  const int ch0 = C1M_CH * (int)blockIdx.y;
  const uint32_t g_first = ((uint32_t)blockIdx.x * 4u + (uint32_t)wave) * (uint32_t)groups_per_wave;
  const uint32_t g_end = min(g_first + (uint32_t)groups_per_wave, ngroups);
  const int word0 = 2 * (int)blockIdx.y;
  // the first patch is requested before the filters are staged, so the two latencies overlap
  // (a wave without pixel groups loads pixel 0's and discards it)
  float xv[27];
  uint32_t inside;
  c1m_issue_patch(x, g_first * 64u + (uint32_t)lane, total_pix, H, W, sH, sW, pH, pW, OH, OW, divOW, divOH, xv, inside);
  const int nch = min(C1M_CH, D - ch0);  // >= 1 by the grid
  c1m_stage_filters(sTap, sSc, sBi, w, scale, bias, ch0, nch, true);
  __syncthreads();  // the only barrier: from here on the waves run independently

  for (uint32_t grp = g_first; grp < g_end; ++grp) {  // wave-uniform bounds
    const uint32_t p = grp * 64u + (uint32_t)lane;
    if (grp != g_first)
      c1m_issue_patch(x, p, total_pix, H, W, sH, sW, pH, pW, OH, OW, divOW, divOH, xv, inside);
#pragma unroll
    for (int k = 0; k < 27; ++k) xv[k] = ((inside >> (k % 9)) & 1u) ? xv[k] : 0.0f;
    uint32_t gw[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int g = 0; g < C1M_CH / 32; ++g) {
      if (32 * g >= nch) break;  // workgroup-uniform: groups past the last channel keep zero bits
      const c1m_v32f acc = c1m_chain(sTap + 32 * g + l32, xv);
      gw[g] = c1m_sign_bits(acc, sSc, sBi, g, half);
    }
    if (p < total_pix) {
      uint64_t *o = outp + (size_t)p * cw_out + word0;
      o[0] = ((uint64_t)gw[1] << 32) | gw[0];
      if (word0 + 1 < cw_out) o[1] = ((uint64_t)gw[3] << 32) | gw[2];
    }
  }
}

// fp32 NCHW output (the map itself, with the affine map if has_affine), same chains, no pipelining.
__global__ __launch_bounds__(256) void conv2d_f32_k27_mfma_kernel(const float *__restrict__ x,
                                                                  const float *__restrict__ w, int H, int W, int D,
                                                                  int sH, int sW, int pH, int pW, int OH, int OW,
                                                                  const float *__restrict__ scale,
                                                                  const float *__restrict__ bias, FastDiv divOW,
                                                                  FastDiv divOH, uint32_t total_pix, uint32_t ngroups,
                                                                  int groups_per_wave, float *__restrict__ outf,
                                                                  int has_affine) {
  __shared__ float sTap[27 * C1M_RS];
  __shared__ float sSc[C1M_CH], sBi[C1M_CH];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int half = lane >> 5, l32 = lane & 31;
  const int ch0 = C1M_CH * (int)blockIdx.y;
  const int nch = min(C1M_CH, D - ch0);  // >= 1 by the grid
  c1m_stage_filters(sTap, sSc, sBi, w, scale, bias, ch0, nch, has_affine != 0);
  __syncthreads();  // the only barrier

  const size_t ohw = (size_t)OH * OW;
  const uint32_t g_first = ((uint32_t)blockIdx.x * 4u + (uint32_t)wave) * (uint32_t)groups_per_wave;
  for (int gi = 0; gi < groups_per_wave; ++gi) {
    const uint32_t grp = g_first + (uint32_t)gi;
    if (grp >= ngroups) break;  // wave-uniform
    float xv[27];
    uint32_t inside;
    c1m_issue_patch(x, grp * 64u + (uint32_t)lane, total_pix, H, W, sH, sW, pH, pW, OH, OW, divOW, divOH, xv, inside);
#pragma unroll
    for (int k = 0; k < 27; ++k) xv[k] = ((inside >> (k % 9)) & 1u) ? xv[k] : 0.0f;
    // NCHW offsets of (image, channel 0, pixel) for the two pixels this lane holds results of
    size_t obase[2];
    bool ov[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const uint32_t q = grp * 64u + 32u * (uint32_t)b + (uint32_t)l32;
      ov[b] = q < total_pix;
      const uint32_t qc = ov[b] ? q : 0u;
      const uint32_t qn = fdiv(fdiv(qc, divOW), divOH);
      obase[b] = (size_t)qn * D * ohw + ((size_t)qc - (size_t)qn * ohw);
    }
#pragma unroll 1
    for (int g = 0; g < C1M_CH / 32; ++g) {
      if (32 * g >= nch) break;  // workgroup-uniform
      const c1m_v32f acc = c1m_chain(sTap + 32 * g + l32, xv);
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int rr = 0; rr < 16; ++rr) {
          const int chl = 32 * g + 8 * (rr >> 2) + 4 * half + (rr & 3);
          if (chl < nch && ov[b]) {
            const float a = acc[16 * b + rr];
            outf[obase[b] + (size_t)(ch0 + chl) * ohw] = has_affine ? fmaf(sSc[chl], a, sBi[chl]) : a;
          }
        }
    }
  }
}

// Launch shape of the matrix-core first layer: one wave per `*gpw` groups of 64 pixels (enough
// groups per wave to amortise the filter staging, enough waves to give every SIMD two).
static dim3 c1m_grid(int64_t total_pix, int D, int *gpw, int64_t wave_slots = 2048) {
  const int64_t ngroups = (total_pix + 63) / 64;
  int64_t g = ngroups / wave_slots;
  g = g < 1 ? 1 : (g > 8 ? 8 : g);
  *gpw = (int)g;
  const int64_t waves = (ngroups + g - 1) / g;
  return dim3((unsigned)((waves + 3) / 4), (unsigned)((D + C1M_CH - 1) / C1M_CH));
}

// Filter bank of a fully-connected layer whose input is a flattened NCHW map [C, H, W],
// re-ordered to the packed NHWC bit order (h, w, c) of the activations: a common
// permutation of the reduction axis leaves the result unchanged.
__global__ __launch_bounds__(256) void pack_fc_weight_nhwc_kernel(const float *__restrict__ w, int C, int HW, int Cw,
                                                                  uint64_t *__restrict__ out, int64_t total_words) {
  const int lane = threadIdx.x & 63;
  const int64_t g = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (g >= total_words) return;
  const int cw = (int)(g % Cw);
  const int hw = (int)((g / Cw) % HW);
  const int64_t n = g / ((int64_t)Cw * HW);
  const int c = cw * 64 + lane;
  float v = -1.0f;
  if (c < C) v = w[(n * C + c) * HW + hw];
  const uint64_t m = __ballot(v >= 0.0f);
  if (lane == 0) out[g] = m;
}

}  // namespace bnn

using namespace bnn;

static bnn_status conv2d_impl(const float *x, const uint64_t *w_packed, int N, int C, int H, int W, int D, int kH,
                              int kW, int sH, int sW, int pH, int pW, int32_t *out_i32, float *out_f32,
                              const float *scale, const float *bias, void *workspace, size_t workspace_bytes,
                              void *stream, const GemmTune &tune) {
  bnn_status st = check_conv_geometry(N, C, H, W, kH, kW, sH, sW, pH, pW);
  if (st != BNN_OK) return st;
  if (D < 0) return BNN_ERR_SHAPE;
  if (N == 0 || D == 0) return BNN_OK;
  if (!x || !w_packed || !workspace || (!out_i32 && !out_f32)) return BNN_ERR_NULL;
  if (out_f32 && (!scale || !bias)) return BNN_ERR_NULL;
  if (!aligned16(x) || !aligned16(w_packed) || !aligned16(workspace) || (out_i32 && !aligned16(out_i32)) ||
      (out_f32 && !aligned16(out_f32)))
    return BNN_ERR_ALIGN;
  const size_t need = bnn_conv2d_workspace_bytes(N, C, H, W, kH, kW, sH, sW, pH, pW);
  if (workspace_bytes < need) return BNN_ERR_WORKSPACE;
  st = conv_limits(N, C, H, W, D, kH, kW, sH, sW, pH, pW);
  if (st != BNN_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  uint64_t *img = reinterpret_cast<uint64_t *>(workspace);
  if (kH == 1 && kW == 1 && pH == 0 && pW == 0) {
    // no patch expansion: encode only the sampled pixels, then a stride-1 1x1 problem on them
    const int OH = (int)bnn_conv_out_dim(H, 1, sH, 0), OW = (int)bnn_conv_out_dim(W, 1, sW, 0);
    st = launch_encode_nchw(x, N, C, H, W, OH, OW, sH, sW, img, s);
    if (st != BNN_OK) return st;
    return conv_from_packed(img, w_packed, N, C, OH, OW, D, 1, 1, 1, 1, 0, 0, 0, out_i32, out_f32, nullptr, scale,
                            bias, s, tune);
  }
  st = launch_encode_nchw(x, N, C, H, W, H, W, 1, 1, img, s);
  if (st != BNN_OK) return st;
  return conv_from_packed(img, w_packed, N, C, H, W, D, kH, kW, sH, sW, pH, pW, 0, out_i32, out_f32, nullptr, scale,
                          bias, s, tune);
}

extern "C" bnn_status bnn_conv2d(const float *x, const uint64_t *w_packed, int N, int C, int H, int W, int D, int kH,
                                 int kW, int sH, int sW, int pH, int pW, int32_t *out_i32, float *out_f32,
                                 const float *scale, const float *bias, void *workspace, size_t workspace_bytes,
                                 void *stream) {
  return conv2d_impl(x, w_packed, N, C, H, W, D, kH, kW, sH, sW, pH, pW, out_i32, out_f32, scale, bias, workspace,
                     workspace_bytes, stream, GemmTune());
}

// ---- bnn_conv2d for callers that cannot allocate ---------------------------------------------
// The packed image goes to a fixed array in device memory instead of a caller workspace.  Every
// GPU the library runs on holds its own copy of the array (at its own address) until the process
// ends.  In host code the array's name is only a handle: its device address is looked up once per
// device, with that device current, and from then on only that address is used.
static __device__ __align__(256) unsigned char scratch[BNN_CONV2D_NOALLOC_MAX_BYTES];

namespace {
constexpr int NOALLOC_MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[NOALLOC_MAX_DEVICES] = {nullptr};

// Device address of `scratch` on the current device, or nullptr on failure.
void *scratch_address() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= NOALLOC_MAX_DEVICES) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}
}  // namespace

extern "C" size_t bnn_conv2d_noalloc_max_bytes(void) { return BNN_CONV2D_NOALLOC_MAX_BYTES; }

extern "C" bnn_status bnn_conv2d_noalloc(const float *x, const uint64_t *w_packed, int N, int C, int H, int W, int D,
                                         int kH, int kW, int sH, int sW, int pH, int pW, int32_t *out_i32,
                                         float *out_f32, const float *scale, const float *bias, void *stream) {
  // the size check comes first and needs no device: a request over the limit never reaches HIP
  bnn_status st = check_conv_geometry(N, C, H, W, kH, kW, sH, sW, pH, pW);
  if (st != BNN_OK) return st;
  if (D < 0) return BNN_ERR_SHAPE;
  if (N == 0 || D == 0) return BNN_OK;
  const size_t need = bnn_conv2d_workspace_bytes(N, C, H, W, kH, kW, sH, sW, pH, pW);
  if (need > BNN_CONV2D_NOALLOC_MAX_BYTES) return BNN_ERR_WORKSPACE;
  if (!x || !w_packed || (!out_i32 && !out_f32)) return BNN_ERR_NULL;
  if (out_f32 && (!scale || !bias)) return BNN_ERR_NULL;
  if (!aligned16(x) || !aligned16(w_packed) || (out_i32 && !aligned16(out_i32)) || (out_f32 && !aligned16(out_f32)))
    return BNN_ERR_ALIGN;
  void *ptr = scratch_address();
  if (!ptr) return BNN_ERR_HIP;
  return conv2d_impl(x, w_packed, N, C, H, W, D, kH, kW, sH, sW, pH, pW, out_i32, out_f32, scale, bias, ptr,
                     BNN_CONV2D_NOALLOC_MAX_BYTES, stream, GemmTune());
}

// Declared in bnn_testing.h.
extern "C" bnn_status bnn_testing_conv2d(const float *x, const uint64_t *w_packed, int N, int C, int H, int W, int D,
                                         int kH, int kW, int sH, int sW, int pH, int pW, int32_t *out_i32,
                                         float *out_f32, const float *scale, const float *bias, void *workspace,
                                         size_t workspace_bytes, int cfg, int lean, void *stream) {
  GemmTune tune;
  tune.cfg = cfg;
  tune.lean = lean;
  return conv2d_impl(x, w_packed, N, C, H, W, D, kH, kW, sH, sW, pH, pW, out_i32, out_f32, scale, bias, workspace,
                     workspace_bytes, stream, tune);
}

static bnn_status conv2d_packed_impl(const uint64_t *x_packed, const uint64_t *w_packed, int N, int C, int H, int W,
                                     int D, int kH, int kW, int sH, int sW, int pH, int pW, int pool,
                                     int32_t *out_i32, float *out_f32, uint64_t *out_packed, const float *scale,
                                     const float *bias, void *stream, const GemmTune &tune) {
  bnn_status st = check_conv_geometry(N, C, H, W, kH, kW, sH, sW, pH, pW);
  if (st != BNN_OK) return st;
  if (D < 0 || (pool != 0 && pool != 2)) return BNN_ERR_SHAPE;
  const int64_t OH = bnn_conv_out_dim(H, kH, sH, pH), OW = bnn_conv_out_dim(W, kW, sW, pW);
  if (pool == 2 && ((OH & 1) || (OW & 1))) return BNN_ERR_SHAPE;
  if (N == 0 || D == 0) return BNN_OK;
  if (!x_packed || !w_packed || (!out_i32 && !out_f32 && !out_packed)) return BNN_ERR_NULL;
  if ((out_f32 || out_packed) && (!scale || !bias)) return BNN_ERR_NULL;
  if (out_packed && (out_i32 || out_f32)) return BNN_ERR_UNSUPPORTED;  // one kind of output per call
  if (pool == 2 && !out_packed) return BNN_ERR_UNSUPPORTED;            // pooling lives in the packed epilogue
  if (!aligned16(x_packed) || !aligned16(w_packed) || (out_i32 && !aligned16(out_i32)) ||
      (out_f32 && !aligned16(out_f32)) || (out_packed && !aligned16(out_packed)))
    return BNN_ERR_ALIGN;
  st = conv_limits(N, C, H, W, D, kH, kW, sH, sW, pH, pW);
  if (st != BNN_OK) return st;
  return conv_from_packed(x_packed, w_packed, N, C, H, W, D, kH, kW, sH, sW, pH, pW, pool, out_i32, out_f32,
                          out_packed, scale, bias, (hipStream_t)stream, tune);
}

extern "C" bnn_status bnn_conv2d_packed(const uint64_t *x_packed, const uint64_t *w_packed, int N, int C, int H, int W,
                                        int D, int kH, int kW, int sH, int sW, int pH, int pW, int pool,
                                        int32_t *out_i32, float *out_f32, uint64_t *out_packed, const float *scale,
                                        const float *bias, void *stream) {
  return conv2d_packed_impl(x_packed, w_packed, N, C, H, W, D, kH, kW, sH, sW, pH, pW, pool, out_i32, out_f32,
                            out_packed, scale, bias, stream, GemmTune());
}

// Declared in bnn_testing.h.
extern "C" bnn_status bnn_testing_conv2d_packed(const uint64_t *x_packed, const uint64_t *w_packed, int N, int C,
                                                int H, int W, int D, int kH, int kW, int sH, int sW, int pH, int pW,
                                                int pool, int32_t *out_i32, float *out_f32, uint64_t *out_packed,
                                                const float *scale, const float *bias, int cfg, int lean,
                                                void *stream) {
  GemmTune tune;
  tune.cfg = cfg;
  tune.lean = lean;
  return conv2d_packed_impl(x_packed, w_packed, N, C, H, W, D, kH, kW, sH, sW, pH, pW, pool, out_i32, out_f32,
                            out_packed, scale, bias, stream, tune);
}

extern "C" bnn_status bnn_conv2d_f32_sign(const float *x, const float *w, int N, int C, int H, int W, int D, int kH,
                                          int kW, int sH, int sW, int pH, int pW, const float *scale,
                                          const float *bias, uint64_t *out_packed, void *stream) {
  bnn_status st = check_conv_geometry(N, C, H, W, kH, kW, sH, sW, pH, pW);
  if (st != BNN_OK) return st;
  if (D < 0) return BNN_ERR_SHAPE;
  if (N == 0 || D == 0) return BNN_OK;
  if (!x || !w || !scale || !bias || !out_packed) return BNN_ERR_NULL;
  if (!aligned16(x) || !aligned16(w) || !aligned16(out_packed)) return BNN_ERR_ALIGN;
  const int64_t K = (int64_t)C * kH * kW;
  if (K > F32S_KMAX) return BNN_ERR_UNSUPPORTED;
  const int64_t OH = bnn_conv_out_dim(H, kH, sH, pH), OW = bnn_conv_out_dim(W, kW, sW, pW);
  const int64_t total = (int64_t)N * OH * OW;
  if (total > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  {
    ProfScope ps(KID_CONV_F32_SIGN, s);
    const dim3 block(256);
    if (K == 27 && C == 3 && kH == 3 && kW == 3) {
      int gpw;
      const dim3 grid = c1m_grid(total, D, &gpw, 4096);  // four resident waves per SIMD
      const uint32_t ngroups = (uint32_t)((total + 63) / 64);
      const int cw = (int)bnn_packed_words(D);
      const FastDiv dOW((uint32_t)OW), dOH((uint32_t)OH);
      hipLaunchKernelGGL(conv2d_f32_k27_mfma_sign_kernel, grid, block, 0, s, x, w, H, W, D, sH, sW, pH, pW, (int)OH,
                         (int)OW, scale, bias, out_packed, cw, dOW, dOH, (uint32_t)total, ngroups, gpw);
    } else {
      const dim3 grid((unsigned)((total + 255) / 256));
      hipLaunchKernelGGL(conv2d_f32_sign_kernel<0>, grid, block, 0, s, x, w, C, H, W, D, kH, kW, sH, sW, pH, pW,
                         (int)OH, (int)OW, scale, bias, out_packed, (int)bnn_packed_words(D), FastDiv((uint32_t)OW),
                         FastDiv((uint32_t)OH), (uint32_t)total, (int)K);
    }
  }
  return launch_status();
}

namespace bnn {
// 3x3x3 real-valued convolution with fp32 NCHW output on the kernel above (arguments validated by
// the caller; scale and bias both given or both null).
bnn_status launch_conv2d_f32_k27(const float *x, const float *w, int N, int H, int W, int D, int sH, int sW, int pH,
                                 int pW, const float *scale, const float *bias, float *out, hipStream_t s) {
  const int64_t OH = bnn_conv_out_dim(H, 3, sH, pH), OW = bnn_conv_out_dim(W, 3, sW, pW);
  const int64_t total = (int64_t)N * OH * OW;
  int gpw;
  const dim3 grid = c1m_grid(total, D, &gpw), block(256);
  hipLaunchKernelGGL(conv2d_f32_k27_mfma_kernel, grid, block, 0, s, x, w, H, W, D, sH, sW, pH, pW, (int)OH, (int)OW,
                     scale, bias, FastDiv((uint32_t)OW), FastDiv((uint32_t)OH), (uint32_t)total,
                     (uint32_t)((total + 63) / 64), gpw, out, scale ? 1 : 0);
  return launch_status();
}
}  // namespace bnn

extern "C" bnn_status bnn_pack_fc_weight_nhwc(const float *w, int64_t Nout, int C, int H, int W, uint64_t *w_packed,
                                              void *stream) {
  if (Nout < 0 || C <= 0 || H <= 0 || W <= 0) return BNN_ERR_SHAPE;
  if (Nout == 0) return BNN_OK;
  if (!w || !w_packed) return BNN_ERR_NULL;
  if (!aligned16(w) || !aligned16(w_packed)) return BNN_ERR_ALIGN;
  const int64_t Cw = bnn_packed_words(C);
  const int64_t HW = (int64_t)H * W;
  if (HW > 0x7fffffffLL || Nout * C * HW > 0x7fffffffLL * 64) return BNN_ERR_UNSUPPORTED;
  const int64_t total = Nout * HW * Cw;
  const int64_t blocks = (total + 3) / 4;
  if (blocks > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  {
    ProfScope ps(KID_PACK_CONV_WEIGHT, s);
    hipLaunchKernelGGL(pack_fc_weight_nhwc_kernel, dim3((unsigned)blocks), dim3(256), 0, s, w, C, (int)HW, (int)Cw,
                       w_packed, total);
  }
  return launch_status();
}
