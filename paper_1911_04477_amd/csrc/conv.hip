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
#include "common.h"

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
                                   hipStream_t s) {
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
  return run_gemm(p, 1, out_packed ? 1 : 0, s);
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

// 3x3x3 specialization (K = 27).  A workgroup computes 64 output channels (one stored word) of
// its pixels; each lane owns F32S_NP output pixels (p + q * part), so one
// set of scalar weight loads feeds 27 * F32S_NP fused multiply-adds, and the loads of the next channel
// (27 weights, scale, bias: 29 SGPRs) are issued before the current channel is computed: the
// scalar-memory latency is covered by compute instead of being waited for per channel.
// Channels run from high to low inside each group of 32, so the sign bit is shifted in with a
// single add-with-carry (word = 2*word + bit).  Loads, wait and carry trick are inline asm;
// the last load statement of a set names the first tap of the first pixel as in/out operand, which
// keeps the multiply-adds of the channel being computed behind the loads of the next one.
// Every SGPR an in-flight load will write is an operand of the wait that follows, so it stays
// reserved until the data has arrived.
constexpr int F32S_NP = 2;
using f32s_u32x2 = uint32_t __attribute__((ext_vector_type(2)));
using f32s_u32x8 = uint32_t __attribute__((ext_vector_type(8)));
using f32s_u32x16 = uint32_t __attribute__((ext_vector_type(16)));
struct F32sWSet {
  f32s_u32x16 a;  // taps 0..15
  f32s_u32x8 b;   // taps 16..23
  f32s_u32x2 c;   // taps 24, 25
  uint32_t d;     // tap 26
  uint32_t sc, bi;
};

__device__ __forceinline__ uint64_t f32s_uniform64(const void *ptr) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)ptr);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uintptr_t)ptr >> 32));
  return ((uint64_t)hi << 32) | (uint64_t)lo;
}

#define F32S_LOAD(S, ch)                                                                                   \
  do {                                                                                                     \
    const uint32_t ch_ = (uint32_t)__builtin_amdgcn_readfirstlane((int)(ch));                              \
    const uint32_t o0_ = ch_ * 108u, o1_ = o0_ + 0x40u, o2_ = o0_ + 0x60u, o3_ = o0_ + 0x68u;              \
    const uint32_t o4_ = ch_ * 4u;                                                                         \
    asm volatile("s_load_dwordx16 %0, %1, %2" : "=s"(S.a) : "s"(wbase), "s"(o0_));                         \
    asm volatile("s_load_dwordx8 %0, %1, %2" : "=s"(S.b) : "s"(wbase), "s"(o1_));                          \
    asm volatile("s_load_dwordx2 %0, %1, %2" : "=s"(S.c) : "s"(wbase), "s"(o2_));                          \
    asm volatile("s_load_dword %0, %1, %2" : "=s"(S.d) : "s"(wbase), "s"(o3_));                            \
    asm volatile("s_load_dword %0, %1, %2" : "=s"(S.sc) : "s"(sbase), "s"(o4_));                           \
    asm volatile("s_load_dword %0, %2, %3" : "=s"(S.bi), "+v"(xv[0][0]) : "s"(bbase), "s"(o4_));           \
  } while (0)
#define F32S_WAIT(S) \
  asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(S.a), "+s"(S.b), "+s"(S.c), "+s"(S.d), "+s"(S.sc), "+s"(S.bi))

// PACK = 1: packed signs of fma(scale, acc, bias) (outp).  PACK = 0: the real-valued map itself,
// fp32 NCHW (outf), fma(scale, acc, bias) if has_affine, else acc.
template <int PACK>
__global__ __launch_bounds__(256) void conv2d_f32_sign27_kernel(const float *__restrict__ x, const float *w_, int H,
                                                                int W, int D, int sH, int sW, int pH, int pW,
                                                                int OH, int OW, const float *scale_,
                                                                const float *bias_, uint64_t *__restrict__ outp,
                                                                int cw_out, FastDiv divOW, FastDiv divOH,
                                                                uint32_t total_pix, uint32_t part,
                                                                float *__restrict__ outf, int has_affine) {
  const uint32_t gid = blockIdx.x * 256u + threadIdx.x;
  const uint64_t wbase = f32s_uniform64(w_), sbase = f32s_uniform64(scale_), bbase = f32s_uniform64(bias_);
  // pixel q of this lane: gid + q * part (the later ones may not exist)
  float xv[F32S_NP][27];
  bool pv[F32S_NP];
  size_t obase[F32S_NP];  // PACK = 0: element offset of (n, channel 0, oh, ow) in the NCHW output
  const size_t ohw = (size_t)OH * OW;
#pragma unroll
  for (int q = 0; q < F32S_NP; ++q) {
    const uint32_t p = gid + (uint32_t)q * part;
    pv[q] = gid < part && p < total_pix;
    const uint32_t pc = pv[q] ? p : 0u;
    const uint32_t t = fdiv(pc, divOW);
    const uint32_t ow = pc - t * OW;
    const uint32_t n = fdiv(t, divOH);
    const uint32_t oh = t - n * OH;
    obase[q] = (size_t)n * D * ohw + (size_t)oh * OW + ow;
    const int ih0 = (int)(oh * sH) - pH, iw0 = (int)(ow * sW) - pW;
    const float *xn = x + (size_t)n * 3 * H * W;
    // Row / column validity once; every tap is loaded unconditionally from a clamped (always
    // readable) position and zeroed afterwards: 27 independent loads, three instructions each.
    bool rok[3], cok[3];
    int roff[3], coff[3];
#pragma unroll
    for (int j = 0; j < 3; ++j) {
      const int ih = ih0 + j, iw = iw0 + j;
      rok[j] = pv[q] && ih >= 0 && ih < H;
      cok[j] = iw >= 0 && iw < W;
      roff[j] = (ih < 0 ? 0 : (ih >= H ? H - 1 : ih)) * W;
      coff[j] = iw < 0 ? 0 : (iw >= W ? W - 1 : iw);
    }
    float raw[27];
#pragma unroll
    for (int k = 0; k < 27; ++k) {
      const int c = k / 9, r = k % 9;
      raw[k] = xn[(size_t)c * H * W + roff[r / 3] + coff[r % 3]];
    }
#pragma unroll
    for (int k = 0; k < 27; ++k) {
      const int r = k % 9;
      xv[q][k] = (rok[r / 3] && cok[r % 3]) ? raw[k] : 0.0f;
    }
  }
  uint32_t word[F32S_NP], hi[F32S_NP];
#pragma unroll
  for (int q = 0; q < F32S_NP; ++q) word[q] = hi[q] = 0u;
  auto compute = [&](const F32sWSet &S, int ch) {
    const float sc = __uint_as_float(S.sc), bi = __uint_as_float(S.bi);
    // the pixels' chains advance together: every multiply-add has independent neighbours
    float acc[F32S_NP];
#pragma unroll
    for (int q = 0; q < F32S_NP; ++q) acc[q] = 0.0f;
#pragma unroll
    for (int k = 0; k < 27; ++k) {
      const float wk = __uint_as_float(k < 16 ? S.a[k & 15] : k < 24 ? S.b[k & 7] : k < 26 ? S.c[k & 1] : S.d);
#pragma unroll
      for (int q = 0; q < F32S_NP; ++q) acc[q] = fmaf(xv[q][k], wk, acc[q]);
    }
    if constexpr (PACK == 0) {
      if (ch < D) {
#pragma unroll
        for (int q = 0; q < F32S_NP; ++q)
          if (pv[q]) outf[obase[q] + (size_t)ch * ohw] = has_affine ? fmaf(sc, acc[q], bi) : acc[q];
      }
      return;
    }
#pragma unroll
    for (int q = 0; q < F32S_NP; ++q) {
      const float y = fmaf(sc, acc[q], bi);
      // word = 2 * word + (y >= 0)
      asm("v_cmp_le_f32 vcc, 0, %1\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc" : "+v"(word[q]) : "v"(y) : "vcc");
    }
    if ((ch & 31) == 0) {
      // a group of 32 channels is complete: drop the bits of channels past D, emit
      const int g = ch >> 5;
      const int left = D - ch;  // real channels in this group
      const uint32_t vm = left >= 32 ? 0xffffffffu : ((1u << left) - 1u);
#pragma unroll
      for (int q = 0; q < F32S_NP; ++q) {
        const uint32_t wv = left > 0 ? (word[q] & vm) : 0u;
        if (g & 1) {
          hi[q] = wv;  // channels descend: the upper half of a word is finished first
        } else {
          const uint32_t p = gid + (uint32_t)q * part;
          if (pv[q]) outp[(size_t)p * cw_out + (g >> 1)] = ((uint64_t)hi[q] << 32) | wv;
        }
        word[q] = 0u;
      }
    }
  };
  // blockIdx.y selects the 64 output channels (one stored word per pixel) this workgroup computes
  const int ch_lo = 64 * (int)blockIdx.y, ch_hi = ch_lo + 63;
  const int last = D - 1;
  F32sWSet SA, SB;
  F32S_LOAD(SA, (ch_hi < last ? ch_hi : last));
  for (int ch = ch_hi; ch > ch_lo; ch -= 2) {
    F32S_WAIT(SA);
    F32S_LOAD(SB, (ch - 1 < last ? ch - 1 : last));
    compute(SA, ch);
    F32S_WAIT(SB);
    if (ch - 2 >= ch_lo) F32S_LOAD(SA, (ch - 2 < last ? ch - 2 : last));
    compute(SB, ch - 1);
  }
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

extern "C" bnn_status bnn_conv2d(const float *x, const uint64_t *w_packed, int N, int C, int H, int W, int D, int kH,
                                 int kW, int sH, int sW, int pH, int pW, int32_t *out_i32, float *out_f32,
                                 const float *scale, const float *bias, void *workspace, size_t workspace_bytes,
                                 void *stream) {
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
                            bias, s);
  }
  st = launch_encode_nchw(x, N, C, H, W, H, W, 1, 1, img, s);
  if (st != BNN_OK) return st;
  return conv_from_packed(img, w_packed, N, C, H, W, D, kH, kW, sH, sW, pH, pW, 0, out_i32, out_f32, nullptr, scale,
                          bias, s);
}

extern "C" bnn_status bnn_conv2d_packed(const uint64_t *x_packed, const uint64_t *w_packed, int N, int C, int H, int W,
                                        int D, int kH, int kW, int sH, int sW, int pH, int pW, int pool,
                                        int32_t *out_i32, float *out_f32, uint64_t *out_packed, const float *scale,
                                        const float *bias, void *stream) {
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
                          out_packed, scale, bias, (hipStream_t)stream);
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
      const int64_t part = (total + F32S_NP - 1) / F32S_NP;
      const dim3 grid((unsigned)((part + 255) / 256), (unsigned)bnn_packed_words(D));
      hipLaunchKernelGGL(conv2d_f32_sign27_kernel<1>, grid, block, 0, s, x, w, H, W, D, sH, sW, pH, pW, (int)OH,
                         (int)OW, scale, bias, out_packed, (int)bnn_packed_words(D), FastDiv((uint32_t)OW),
                         FastDiv((uint32_t)OH), (uint32_t)total, (uint32_t)part, (float *)nullptr, 1);
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
  const int64_t part = (total + F32S_NP - 1) / F32S_NP;
  const dim3 grid((unsigned)((part + 255) / 256), (unsigned)bnn_packed_words(D)), block(256);
  // without an affine map the kernel still issues its (unused) scalar loads of scale and bias:
  // point them at readable memory
  hipLaunchKernelGGL(conv2d_f32_sign27_kernel<0>, grid, block, 0, s, x, w, H, W, D, sH, sW, pH, pW, (int)OH, (int)OW,
                     scale ? scale : w, bias ? bias : w, (uint64_t *)nullptr, (int)bnn_packed_words(D),
                     FastDiv((uint32_t)OW), FastDiv((uint32_t)OH), (uint32_t)total, (uint32_t)part, out,
                     scale ? 1 : 0);
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
