// The paper's fp32 "control group" (section 4.4): the same binarized convolution computed the
// ordinary way, as a real-valued GEMM on sign(x) and sign(w), so that the speed-up of the
// Xnor-Bitcount kernel can be restated on this machine.  Not part of the method.
//
// It is given a fair chance: an implicit GEMM (no fp32 patch matrix is written) on the fp32
// matrix cores, V_MFMA_F32_32X32X2F32.  C[d, n] = sum_k sign(w[d, k]) * sign(patch(n)[k]) with
// k = (c, kh, kw) as in the stock im2col order of section 2.1; taps outside the image are
// sign(0) = +1.  All products and partial sums are integers below 2^24, so every fp32
// summation order gives the same, exact result and the output equals the binarized path's.
//
// Workgroup: 256 threads = 2 x 2 waves, tile 128 (output channels) x 128 (pixels), K in chunks
// of 16.  Both operand tiles are staged through double-buffered LDS k-major ([k][row], row
// stride 132 floats), so that an MFMA operand (lane l: row l % 32, k = l / 32) is one
// conflict-free 4-byte LDS read.  A wave owns 64 x 64: 2 x 2 blocks of 32 x 32.
#include "common.h"

namespace bnn {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int CT_BM = 128, CT_BN = 128, CT_BK = 16, CT_RS = 132;

struct ControlParams {
  const float *x, *w;
  float *out;
  int N, C, H, W, D, kH, kW, sH, sW, pH, pW, OH, OW;
  int K;            // C * kH * kW
  int P;            // N * OH * OW
  int tilesM;
  FastDiv divOW, divOH, divTaps, divKW;
};

__device__ __forceinline__ float sign_pm1(float v) { return v >= 0.0f ? 1.0f : -1.0f; }

__global__ __launch_bounds__(256) void control_conv_f32_mfma_kernel(ControlParams p) {
  __shared__ float sA[2][CT_BK * CT_RS];
  __shared__ float sB[2][CT_BK * CT_RS];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int mi = blockIdx.x % p.tilesM, ni = blockIdx.x / p.tilesM;
  const int m0 = mi * CT_BM, n0 = ni * CT_BN;

  // ---- staging roles ------------------------------------------------------------------
  // A (weights): thread t reads 4 consecutive k of row (t / 4) and of row (t / 4 + 64).
  const int a_row = tid >> 2, a_k4 = (tid & 3) * 4;
  // B (patches): thread t owns pixel (t % 128) and the k values (t / 128) * 8 .. + 7 of a chunk;
  // consecutive lanes are consecutive pixels, so the 4-byte loads of a tap coalesce.
  const int b_pix = tid & 127, b_k8 = (tid >> 7) * 8;
  const int n = n0 + b_pix;
  const bool n_ok = n < p.P;
  const uint32_t nn = n_ok ? (uint32_t)n : 0u;
  const uint32_t t1 = fdiv(nn, p.divOW);
  const int ow = (int)(nn - t1 * (uint32_t)p.OW);
  const uint32_t img = fdiv(t1, p.divOH);
  const int oh = (int)(t1 - img * (uint32_t)p.OH);
  const int ih0 = oh * p.sH - p.pH, iw0 = ow * p.sW - p.pW;
  const float *ximg = p.x + (size_t)img * p.C * p.H * p.W;
  const int taps = p.kH * p.kW;

  // load_tiles only ISSUES the loads (unconditional, from clamped positions, so none waits for
  // another); sign, masking and the LDS writes happen in store_tiles, after the current chunk's
  // matrix instructions have been issued.
  float ra[2][4], rb[8];
  uint32_t va = 0, vb = 0, vin = 0;  // element is inside the matrix / the tap is inside the image
  auto load_tiles = [&](int k0) {
    va = vb = vin = 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int m = m0 + a_row + 64 * h;
      const int mc = m < p.D ? m : p.D - 1;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int k = k0 + a_k4 + e;
        const int kc = k < p.K ? k : p.K - 1;
        va |= (uint32_t)(m < p.D && k < p.K) << (4 * h + e);
        ra[h][e] = p.w[(size_t)mc * p.K + kc];
      }
    }
    // (c, kh, kw) of this thread's first k by division, of the following seven by stepping
    const uint32_t kf = (uint32_t)min(k0 + b_k8, p.K - 1);
    int c = (int)fdiv(kf, p.divTaps);
    const uint32_t r0 = kf - (uint32_t)c * (uint32_t)taps;
    int kh = (int)fdiv(r0, p.divKW);
    int kw = (int)(r0 - (uint32_t)kh * (uint32_t)p.kW);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int k = k0 + b_k8 + e;
      const int ih = ih0 + kh, iw = iw0 + kw;
      const bool inside = ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
      const int ihc = ih < 0 ? 0 : (ih >= p.H ? p.H - 1 : ih), iwc = iw < 0 ? 0 : (iw >= p.W ? p.W - 1 : iw);
      vb |= (uint32_t)(n_ok && k < p.K) << e;
      vin |= (uint32_t)inside << e;
      rb[e] = ximg[((size_t)c * p.H + ihc) * p.W + iwc];
      // next k (stops at the last valid one, whose value is then masked by vb)
      if (k + 1 < p.K) {
        if (++kw == p.kW) {
          kw = 0;
          if (++kh == p.kH) {
            kh = 0;
            ++c;
          }
        }
      }
    }
  };
  auto store_tiles = [&](int buf) {
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int e = 0; e < 4; ++e)
        sA[buf][(a_k4 + e) * CT_RS + a_row + 64 * h] = ((va >> (4 * h + e)) & 1u) ? sign_pm1(ra[h][e]) : 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      // a tap outside the image: sign(0) = +1; an element outside the matrix: 0
      const float v = ((vin >> e) & 1u) ? sign_pm1(rb[e]) : 1.0f;
      sB[buf][(b_k8 + e) * CT_RS + b_pix] = ((vb >> e) & 1u) ? v : 0.0f;
    }
  };

  v16f acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;

  const int nchunks = (p.K + CT_BK - 1) / CT_BK;
  load_tiles(0);
  store_tiles(0);
  __syncthreads();
  const int a_off = (lane >> 5) * CT_RS + 64 * wm + (lane & 31);
  const int b_off = (lane >> 5) * CT_RS + 64 * wn + (lane & 31);
  for (int c = 0; c < nchunks; ++c) {
    const int buf = c & 1;
    const bool more = c + 1 < nchunks;
    if (more) load_tiles((c + 1) * CT_BK);
    const float *A = sA[buf], *Bt = sB[buf];
#pragma unroll
    for (int ks = 0; ks < CT_BK / 2; ++ks) {
      float a[2], b[2];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) a[mb] = A[2 * ks * CT_RS + a_off + 32 * mb];
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) b[nb] = Bt[2 * ks * CT_RS + b_off + 32 * nb];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
          acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mb], b[nb], acc[mb][nb], 0, 0, 0);
    }
    if (more) {
      store_tiles(buf ^ 1);  // last read in chunk c - 1, before the previous barrier
      __syncthreads();
    }
  }

  // D[i][j] of a 32 x 32 block: lane l holds column j = l % 32; register r holds row
  // i = 8 * (r / 4) + 4 * (l / 32) + (r % 4).  Scatter to NCHW.
  const int64_t ohw = (int64_t)p.OH * p.OW;
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    const int nc = n0 + 64 * wn + 32 * nb + (lane & 31);
    if (nc >= p.P) continue;
    const uint32_t q1 = fdiv((uint32_t)nc, p.divOW);
    const uint32_t im = fdiv(q1, p.divOH);
    const int64_t pix = (int64_t)nc - (int64_t)im * ohw;
    float *o = p.out + (int64_t)im * p.D * ohw + pix;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + 64 * wm + 32 * mb + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (m < p.D) o[(int64_t)m * ohw] = acc[mb][nb][r];
      }
  }
}

}  // namespace bnn

using namespace bnn;

extern "C" bnn_status bnn_control_conv2d_f32(const float *x, const float *w, int N, int C, int H, int W, int D, int kH,
                                             int kW, int sH, int sW, int pH, int pW, float *out, void *stream) {
  bnn_status st = check_conv_geometry(N, C, H, W, kH, kW, sH, sW, pH, pW);
  if (st != BNN_OK) return st;
  if (D < 0) return BNN_ERR_SHAPE;
  if (N == 0 || D == 0) return BNN_OK;
  if (!x || !w || !out) return BNN_ERR_NULL;
  if (!aligned16(x) || !aligned16(w) || !aligned16(out)) return BNN_ERR_ALIGN;
  const int64_t OH = bnn_conv_out_dim(H, kH, sH, pH), OW = bnn_conv_out_dim(W, kW, sW, pW);
  const int64_t P = (int64_t)N * OH * OW, K = (int64_t)C * kH * kW;
  if (P > 0x7fffff00LL || K > 0xffffffLL || (int64_t)D * K > 0x7fffffffLL * 2) return BNN_ERR_UNSUPPORTED;
  ControlParams p;
  p.x = x; p.w = w; p.out = out;
  p.N = N; p.C = C; p.H = H; p.W = W; p.D = D; p.kH = kH; p.kW = kW; p.sH = sH; p.sW = sW; p.pH = pH; p.pW = pW;
  p.OH = (int)OH; p.OW = (int)OW; p.K = (int)K; p.P = (int)P;
  p.tilesM = (D + CT_BM - 1) / CT_BM;
  p.divOW = FastDiv((uint32_t)OW); p.divOH = FastDiv((uint32_t)OH);
  p.divTaps = FastDiv((uint32_t)(kH * kW)); p.divKW = FastDiv((uint32_t)kW);
  const int64_t blocks = (int64_t)p.tilesM * ((P + CT_BN - 1) / CT_BN);
  if (blocks > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  {
    ProfScope ps(KID_CONTROL_CONV_F32, s);
    hipLaunchKernelGGL(control_conv_f32_mfma_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p);
  }
  return launch_status();
}
