// Packed im2col (section 2.1 im2col applied to the encoded input of section 3.1).
//
// Two streaming passes, both HBM-bound:
//   1. encode_nchw_kernel (encode.hip): fp32 NCHW -> packed NHWC, ceil(C/64) words per
//      pixel.  The fp32 image is read exactly once.
//   2. im2col_gather_kernel (here): every output pixel's kH*kW taps are whole-word
//      copies out of the packed image (which is 32x smaller than the fp32 one and
//      stays in L2), or the "+1" pad word for taps outside the image: zero-padding
//      before the sign makes every real channel of such a tap +1, i.e. bit 1.
// A 1x1 / pad-0 convolution has no patch expansion: pass 1 writes the patch matrix
// directly, sampling the strided pixels.
#include "common.h"

namespace bnn {

bnn_status launch_encode_nchw(const float *x, int N, int C, int H, int W, int OHp, int OWp, int sH, int sW,
                              uint64_t *out, hipStream_t s);

struct GatherParams {
  int C, H, W, OH, OW, kW, sH, sW, pH, pW, Cw;
  FastDiv divRow;   // pieces per patch row
  FastDiv divTap;   // pieces per tap
  FastDiv divKW, divOW, divOH;
  uint32_t total;   // pieces
};

// words of a tap that lies outside the image
__device__ __forceinline__ uint64_t pad_word(int C, int cw) {
  const int left = C - cw * 64;
  return left >= 64 ? ~0ull : (left <= 0 ? 0ull : ((1ull << left) - 1ull));
}

template <int PIECE>  // words per thread: 2 (16-byte copies) or 1
__global__ __launch_bounds__(256) void im2col_gather_kernel(const uint64_t *__restrict__ img,
                                                            uint64_t *__restrict__ cols, GatherParams g) {
  const uint32_t o = blockIdx.x * 256u + threadIdx.x;
  if (o >= g.total) return;
  const uint32_t p = fdiv(o, g.divRow);
  const uint32_t r = o - p * g.divRow.d;
  const uint32_t tap = fdiv(r, g.divTap);
  const uint32_t q = r - tap * g.divTap.d;
  const uint32_t kh = fdiv(tap, g.divKW);
  const uint32_t kw = tap - kh * g.kW;
  const uint32_t t = fdiv(p, g.divOW);
  const uint32_t ow = p - t * g.OW;
  const uint32_t n = fdiv(t, g.divOH);
  const uint32_t oh = t - n * g.OH;
  const int ih = (int)(oh * g.sH + kh) - g.pH;
  const int iw = (int)(ow * g.sW + kw) - g.pW;
  const bool inside = ih >= 0 && ih < g.H && iw >= 0 && iw < g.W;
  if (PIECE == 2) {
    uint4 v;
    if (inside) {
      v = *reinterpret_cast<const uint4 *>(img + (((size_t)n * g.H + ih) * g.W + iw) * g.Cw + 2 * q);
    } else {
      const uint64_t w0 = pad_word(g.C, 2 * q), w1 = pad_word(g.C, 2 * q + 1);
      v.x = (uint32_t)w0; v.y = (uint32_t)(w0 >> 32); v.z = (uint32_t)w1; v.w = (uint32_t)(w1 >> 32);
    }
    reinterpret_cast<uint4 *>(cols)[o] = v;
  } else {
    uint64_t v;
    if (inside) v = img[(((size_t)n * g.H + ih) * g.W + iw) * g.Cw + q];
    else v = pad_word(g.C, q);
    cols[o] = v;
  }
}

static bool conv_geometry_ok(int N, int C, int H, int W, int kH, int kW, int sH, int sW, int pH, int pW) {
  return N >= 0 && C > 0 && H > 0 && W > 0 && kH > 0 && kW > 0 && sH > 0 && sW > 0 && pH >= 0 && pW >= 0 &&
         bnn_conv_out_dim(H, kH, sH, pH) > 0 && bnn_conv_out_dim(W, kW, sW, pW) > 0;
}

static inline size_t round256(size_t b) { return (b + 255) & ~(size_t)255; }

static inline bool is_pointwise(int kH, int kW, int pH, int pW) { return kH == 1 && kW == 1 && pH == 0 && pW == 0; }

// Shared by bnn_im2col_packed and bnn_conv2d; arguments already validated.
bnn_status run_im2col(const float *x, int N, int C, int H, int W, int kH, int kW, int sH, int sW, int pH, int pW,
                      uint64_t *cols, void *workspace, hipStream_t s) {
  const int OH = (int)bnn_conv_out_dim(H, kH, sH, pH), OW = (int)bnn_conv_out_dim(W, kW, sW, pW);
  if (is_pointwise(kH, kW, pH, pW)) return launch_encode_nchw(x, N, C, H, W, OH, OW, sH, sW, cols, s);
  uint64_t *img = reinterpret_cast<uint64_t *>(workspace);
  bnn_status st = launch_encode_nchw(x, N, C, H, W, H, W, 1, 1, img, s);
  if (st != BNN_OK) return st;
  const int Cw = (int)bnn_packed_words(C);
  const int piece = (Cw % 2 == 0) ? 2 : 1;
  const int64_t per_tap = Cw / piece;
  const int64_t per_row = per_tap * kH * kW;
  const int64_t total = (int64_t)N * OH * OW * per_row;
  if (total > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  GatherParams g;
  g.C = C; g.H = H; g.W = W; g.OH = OH; g.OW = OW; g.kW = kW; g.sH = sH; g.sW = sW; g.pH = pH; g.pW = pW;
  g.Cw = Cw;
  g.divRow = FastDiv((uint32_t)per_row);
  g.divTap = FastDiv((uint32_t)per_tap);
  g.divKW = FastDiv((uint32_t)kW);
  g.divOW = FastDiv((uint32_t)OW);
  g.divOH = FastDiv((uint32_t)OH);
  g.total = (uint32_t)total;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  {
    ProfScope ps(KID_IM2COL_GATHER, s);
    if (piece == 2)
      hipLaunchKernelGGL(im2col_gather_kernel<2>, dim3(blocks), dim3(256), 0, s, img, cols, g);
    else
      hipLaunchKernelGGL(im2col_gather_kernel<1>, dim3(blocks), dim3(256), 0, s, img, cols, g);
  }
  return launch_status();
}

bnn_status check_conv_geometry(int N, int C, int H, int W, int kH, int kW, int sH, int sW, int pH, int pW) {
  if (!conv_geometry_ok(N, C, H, W, kH, kW, sH, sW, pH, pW)) return BNN_ERR_SHAPE;
  const int64_t OH = bnn_conv_out_dim(H, kH, sH, pH), OW = bnn_conv_out_dim(W, kW, sW, pW);
  const int64_t Cw = bnn_packed_words(C);
  if ((int64_t)N * C * H * W > 0x7fffffffLL * 4 || (int64_t)N * H * W > 0x7fffffffLL ||
      (int64_t)N * OH * OW * kH * kW * Cw > 0x7fffffffLL || (int64_t)kH * kW > 0x7fff)
    return BNN_ERR_UNSUPPORTED;
  return BNN_OK;
}

}  // namespace bnn

using namespace bnn;

extern "C" size_t bnn_im2col_workspace_bytes(int N, int C, int H, int W, int kH, int kW, int sH, int sW, int pH,
                                             int pW) {
  if (!conv_geometry_ok(N, C, H, W, kH, kW, sH, sW, pH, pW)) return 0;
  if (is_pointwise(kH, kW, pH, pW)) return 0;
  return round256((size_t)N * H * W * (size_t)bnn_packed_words(C) * 8);
}

extern "C" size_t bnn_conv2d_workspace_bytes(int N, int C, int H, int W, int kH, int kW, int sH, int sW, int pH,
                                             int pW) {
  if (!conv_geometry_ok(N, C, H, W, kH, kW, sH, sW, pH, pW)) return 0;
  // the packed image the implicit GEMM gathers from: the whole input, or, for a 1x1 / pad-0
  // convolution, only the pixels its strides sample
  if (is_pointwise(kH, kW, pH, pW)) {
    const size_t OH = (size_t)bnn_conv_out_dim(H, kH, sH, pH), OW = (size_t)bnn_conv_out_dim(W, kW, sW, pW);
    return round256((size_t)N * OH * OW * (size_t)bnn_packed_words(C) * 8);
  }
  return round256((size_t)N * H * W * (size_t)bnn_packed_words(C) * 8);
}

extern "C" bnn_status bnn_im2col_packed(const float *x, int N, int C, int H, int W, int kH, int kW, int sH, int sW,
                                        int pH, int pW, uint64_t *cols, void *workspace, size_t workspace_bytes,
                                        void *stream) {
  bnn_status st = check_conv_geometry(N, C, H, W, kH, kW, sH, sW, pH, pW);
  if (st != BNN_OK) return st;
  if (N == 0) return BNN_OK;
  const size_t need = bnn_im2col_workspace_bytes(N, C, H, W, kH, kW, sH, sW, pH, pW);
  if (!x || !cols || (need > 0 && !workspace)) return BNN_ERR_NULL;
  if (!aligned16(x) || !aligned16(cols) || (need > 0 && !aligned16(workspace))) return BNN_ERR_ALIGN;
  if (workspace_bytes < need) return BNN_ERR_WORKSPACE;
  return run_im2col(x, N, C, H, W, kH, kW, sH, sW, pH, pW, cols, workspace, (hipStream_t)stream);
}
