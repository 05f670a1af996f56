// Binarized convolution driver: the forward graph of Figure 3 of the paper
// (im2col + encode of the input, pre-encoded weight, Xnor-Bitcount, reshape to the
// output feature map).  The reshape (col2im of section 2.1) costs nothing here: the GEMM
// store writes each accumulator straight to its NCHW position.
#include "common.h"

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
  const int64_t OH = bnn_conv_out_dim(H, kH, sH, pH), OW = bnn_conv_out_dim(W, kW, sW, pW);
  const int64_t P = (int64_t)N * OH * OW;
  const int64_t Kw = bnn_conv_kwords(C, kH, kW);
  if (P > 0x7ffffff0LL || (int64_t)D * 8 * Kw > 0xffffffffLL || (int64_t)D * P > 0x7fffffffLL * 8)
    return BNN_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;

  const size_t img_bytes = bnn_im2col_workspace_bytes(N, C, H, W, kH, kW, sH, sW, pH, pW);
  uint64_t *cols = reinterpret_cast<uint64_t *>(static_cast<char *>(workspace) + img_bytes);
  st = run_im2col(x, N, C, H, W, kH, kW, sH, sW, pH, pW, cols, workspace, s);
  if (st != BNN_OK) return st;

  GemmParams p;
  p.A = reinterpret_cast<const uint32_t *>(w_packed);
  p.B = cols;
  p.lda32 = 2 * Kw;
  p.ldb = Kw;
  p.M = D;
  p.N = (int)P;
  p.Kbits = (int)(Kw * 64);  // pad bits are 0 in both operands: they cancel in the exclusive-or
  p.Kformula = C * kH * kW;
  p.Kd = (int)(Kw * 2);
  p.Kw64 = (int)Kw;
  p.b_vec16 = (Kw % 2 == 0) ? 1 : 0;
  p.C = out_i32;
  p.Y = out_f32;
  p.ldc = p.ldy = OH * OW;
  p.scale = scale;
  p.bias = bias;
  p.axis = BNN_CH_ROW;
  p.OHW = (uint32_t)(OH * OW);
  p.divOHW = FastDiv((uint32_t)(OH * OW));
  p.img_stride = (int64_t)D * OH * OW;
  return run_gemm(p, s);
}
