// Xnor-Bitcount convolution (section 3.2 on the implicit patch matrix of section 2.1) for problems
// with very few output pixels: the latency form.
//
// At a batch of a few images the later layers of a network have tens to hundreds of output
// pixels.  The throughput kernel then launches a handful of workgroups, each of which walks the
// whole reduction axis alone (one 256-bit chunk after the other, a memory round trip and a
// barrier per chunk), three quarters of its lanes idle, and the layer lasts as long as that one
// serial walk.  Here the work is cut the other way:
//   * a tile is 32 output channels x 64 columns, ONE column per lane (no idle register columns),
//     and the reduction axis is split over KS slices: a workgroup is 4 x KS waves (row group x
//     slice), so a layer with 16 tiles still occupies 256 waves and each wave walks 1/KS of K;
//   * no LDS staging and no barrier in the loop: a lane gathers the chunk of its own column
//     straight from the packed NHWC image (tap decode per 16-byte piece; taps outside the image
//     are the "+1" pad word), two chunks ahead; A comes through scalar loads as everywhere else;
//   * partial counts are additive (section 3.2: a sum over the reduction axis): the slices meet
//     in LDS once, at the end, and the slice-0 waves run the epilogue -- int32 / fp32 NCHW, or
//     the binarizing epilogue (optional 2x2 max-pool, affine map, sign) that writes packed NHWC;
//   * with pooling the columns are ordered window-major with the member index in the low two
//     bits (column = 4 * window + member), so the four members of a pooling window sit in four
//     neighbouring lanes and the max is two cross-lane steps.
// Requires an even number of words per pixel (16-byte pieces never straddle a tap, rows end on a
// chunk or half-chunk boundary); the host checks it.
#include "common.h"
#include "gemm_rows.inc"

namespace bnn {

using u32x4 = uint32_t __attribute__((ext_vector_type(4)));
using u32x8 = uint32_t __attribute__((ext_vector_type(8)));

__device__ __forceinline__ uint64_t lat_pad_word64(int C, int cw) {
  const int left = C - cw * 64;
  return left >= 64 ? ~0ull : (left <= 0 ? 0ull : ((1ull << left) - 1ull));
}

template <int KS, int EMODE>
__global__ __launch_bounds__(256 * KS) void xnor_conv_latency_kernel(GemmParams p) {
  constexpr int DEPTH = 2;  // chunks in flight (five, a whole slice at once, measured slower: 15.3 against 12.8 us on the last layer)
  __shared__ int sRed[KS * 4 * 8 * 64];
  __shared__ __attribute__((aligned(16))) uint8_t sO[64 * 4];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave & 3;   // row group of 8 inside the 32-row tile
  const int ks = wave >> 2;  // slice of the reduction axis
  const int mi = (int)(blockIdx.x % (uint32_t)p.tilesM);
  const int ni = (int)(blockIdx.x / (uint32_t)p.tilesM);
  const int m0 = mi * 32 + wm * 8;
  const int n = ni * 64 + lane;
  const ConvGeom &g = p.g;

  // ---- this lane's column -> output pixel ----------------------------------------------------------
  const bool col_ok = n < p.N;
  uint32_t img = 0;
  int oh = 0, ow = 0;
  if (col_ok) {
    if (g.pool == 0) {
      const uint32_t t = fdiv((uint32_t)n, g.divOW);
      ow = (int)((uint32_t)n - t * (uint32_t)g.OW);
      img = fdiv(t, g.divOH);
      oh = (int)(t - img * (uint32_t)g.OH);
    } else {
      const uint32_t j = (uint32_t)n & 3u, wdx = (uint32_t)n >> 2;
      const uint32_t PW = (uint32_t)g.OW >> 1, PH = (uint32_t)g.OH >> 1;
      const uint32_t t = fdiv(wdx, g.divOW);
      const uint32_t wx = wdx - t * PW;
      img = fdiv(t, g.divOH);
      const uint32_t wy = t - img * PH;
      oh = (int)(2 * wy + (j >> 1));
      ow = (int)(2 * wx + (j & 1));
    }
  }
  const int ih0 = oh * g.sH - g.pH, iw0 = ow * g.sW - g.pW;
  const uint64_t *act_img = g.act + (size_t)img * (size_t)(g.H * g.W) * (size_t)g.Cw;

  // one 16-byte piece (words 2e, 2e + 1 of the patch row): both words belong to one tap
  auto gather_piece = [&](int e) -> u32x4 {
    const uint32_t w = 2u * (uint32_t)e;
    u32x4 v = {0u, 0u, 0u, 0u};
    if ((int)w >= p.Kw64 || !col_ok) return v;  // past the row: zero in both operands
    const uint32_t tap = fdiv(w, g.divCw);
    const int cw = (int)(w - tap * (uint32_t)g.Cw);
    const uint32_t kh = fdiv(tap, g.divKW);
    const int kw = (int)(tap - kh * (uint32_t)g.kW);
    const int ih = ih0 + (int)kh, iw = iw0 + kw;
    if (ih >= 0 && ih < g.H && iw >= 0 && iw < g.W) {
      v = *reinterpret_cast<const u32x4 *>(act_img + (size_t)(ih * g.W + iw) * (size_t)g.Cw + cw);
    } else {
      const uint64_t x0 = lat_pad_word64(g.C, cw), x1 = lat_pad_word64(g.C, cw + 1);
      v.x = (uint32_t)x0; v.y = (uint32_t)(x0 >> 32); v.z = (uint32_t)x1; v.w = (uint32_t)(x1 >> 32);
    }
    return v;
  };

  // ---- A: this wave's 8 rows through scalar loads ---------------------------------------------------
  const uint32_t arow_bytes = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)p.lda32 * 4u));
  const uint32_t aoff_max = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)(p.M - 1) * (uint32_t)p.lda32 * 4u));
  const uint32_t aoff_first = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)min(m0, p.M - 1) * (uint32_t)p.lda32 * 4u));
  const uint32_t Abase_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)p.A);
  const uint32_t Abase_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uintptr_t)p.A >> 32));
  const uint64_t Abase0 = ((uint64_t)Abase_hi << 32) | (uint64_t)Abase_lo;
#define BNN_LAT_AOFF(i) min(aoff_first + (uint32_t)(i) * arow_bytes, aoff_max)

  int acc[8][1];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i][0] = 0;

  // ---- this slice's chunks ---------------------------------------------------------------------------
  const int nfull_all = p.Kw64 / 4;            // full chunks of 4 words
  const bool has_half = (p.Kw64 & 3) == 2;     // rows of 4 n + 2 words end with a half chunk
  const int per = (nfull_all + KS - 1) / KS;
  const int cb = min(ks * per, nfull_all);
  const int nfull = min(per, nfull_all - cb);
  auto load_b = [&](u32x8 &b, int cl) {
    const int c = cb + cl;
    b.lo = gather_piece(2 * c);
    b.hi = gather_piece(2 * c + 1);
  };
  auto compute = [&](const u32x8 &bv, int cl) {
    const uint64_t Abase = Abase0 + (uint64_t)(uint32_t)(cb + cl) * 32u;
    u32x8 a[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
      asm volatile("s_load_dwordx8 %0, %1, %2" : "=s"(a[i]) : "s"(Abase), "s"(BNN_LAT_AOFF(i)));
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+s"(a[0]), "+s"(a[1]), "+s"(a[2]), "+s"(a[3]), "+s"(a[4]), "+s"(a[5]), "+s"(a[6]), "+s"(a[7]));
    uint32_t t0, t1;
#define BNN_BV(j, d) bv[d]
#pragma unroll
    for (int i = 0; i < 8; ++i) BNN_GEMM_ROW_1_NY(acc[i], a[i], BNN_BV, t0, t1);
#undef BNN_BV
  };
  u32x8 bq[DEPTH];
#pragma unroll
  for (int d = 0; d < DEPTH; ++d)
    if (d < nfull) load_b(bq[d], d);
  int c = 0;
  for (; c + DEPTH <= nfull; c += DEPTH) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      compute(bq[d], c + d);
      if (c + d + DEPTH < nfull) load_b(bq[d], c + d + DEPTH);
    }
  }
#pragma unroll
  for (int d = 0; d < DEPTH; ++d)
    if (c + d < nfull) compute(bq[d], c + d);
  // the half chunk (last two words), by the last slice
  if (has_half && ks == KS - 1) {
    const u32x4 bv = gather_piece(2 * nfull_all);
    const uint64_t Abase = Abase0 + (uint64_t)(uint32_t)nfull_all * 32u;
    u32x4 a[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
      asm volatile("s_load_dwordx4 %0, %1, %2" : "=s"(a[i]) : "s"(Abase), "s"(BNN_LAT_AOFF(i)));
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+s"(a[0]), "+s"(a[1]), "+s"(a[2]), "+s"(a[3]), "+s"(a[4]), "+s"(a[5]), "+s"(a[6]), "+s"(a[7]));
    uint32_t t0, t1;
#define BNN_BV(j, d) bv[d]
#pragma unroll
    for (int i = 0; i < 8; ++i) BNN_GEMM_HALF_1_NY(acc[i], a[i], BNN_BV, t0, t1);
#undef BNN_BV
  }
#undef BNN_LAT_AOFF

  // ---- slices meet in LDS ----------------------------------------------------------------------------
#pragma unroll
  for (int i = 0; i < 8; ++i) sRed[((ks * 4 + wm) * 8 + i) * 64 + lane] = acc[i][0];
  __syncthreads();
  if (ks == 0) {  // wave-uniform
    int tot[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int t = 0;
#pragma unroll
      for (int k = 0; k < KS; ++k) t += sRed[((k * 4 + wm) * 8 + i) * 64 + lane];
      tot[i] = t;
    }
    if constexpr (EMODE == 0) {
      // int32 and / or fp32, NCHW (columns are pixels in NHWC order: n -> image, pixel)
      if (col_ok) {
        const uint32_t im = fdiv((uint32_t)n, p.divOHW);
        const uint32_t pix = (uint32_t)n - im * p.OHW;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int m = m0 + i;
          if (m < p.M) {
            const int v = p.Kformula - 2 * tot[i];
            const int64_t off = (int64_t)im * p.img_stride + pix;
            if (p.C) p.C[off + (int64_t)m * p.ldc] = v;
            if (p.Y) p.Y[off + (int64_t)m * p.ldy] = fmaf(p.scale[m], (float)v, p.bias[m]);
          }
        }
      }
    } else {
      // binarizing epilogue: K - 2*acc decreases in acc, so the 2x2 max is K - 2*min(acc) over the
      // four neighbouring lanes of a window; rows run from the last to the first so that each sign
      // is shifted in with one add
      uint32_t byte = 0u;
#pragma unroll
      for (int i = 7; i >= 0; --i) {
        const int m = m0 + i;
        const bool row_ok = m < p.M;
        const float sc = row_ok ? p.scale[m] : 0.0f;
        const float bi = row_ok ? p.bias[m] : -1.0f;  // rows past M give bit 0
        int a = tot[i];
        if (g.pool) {
          a = min(a, __shfl_xor(a, 1));
          a = min(a, __shfl_xor(a, 2));
        }
        const float y = fmaf(sc, (float)(p.Kformula - 2 * a), bi);
        byte = 2u * byte + (y >= 0.0f ? 1u : 0u);
      }
      sO[lane * 4 + wm] = (uint8_t)byte;
    }
  }
  if constexpr (EMODE == 1) {
    __syncthreads();
    // one thread per output pixel writes the 32-channel half word of this tile
    const int npix = g.pool ? 16 : 64;
    if (tid < npix) {
      const int colsel = g.pool ? 4 * tid : tid;  // a window's four lanes hold the same byte
      const int64_t gp = g.pool ? (int64_t)ni * 16 + tid : (int64_t)ni * 64 + tid;
      const int64_t limit = g.pool ? (int64_t)(p.N >> 2) : (int64_t)p.N;
      if (gp < limit) {
        const uint32_t w = *reinterpret_cast<const uint32_t *>(&sO[colsel * 4]);
        uint32_t *o32 = reinterpret_cast<uint32_t *>(p.outp) + (gp * p.cw_out) * 2;
        o32[mi] = w;
        if (mi == p.tilesM - 1 && (p.tilesM & 1)) o32[mi + 1] = 0u;  // channels past D: pad bits 0
      }
    }
  }
}

// Whether the latency form can run the implicit GEMM described by p.
bool latency_applicable(const GemmParams &p) {
  if ((p.g.Cw & 1) != 0) return false;                       // 16-byte pieces must not straddle taps
  if (p.Kw64 != p.g.kH * p.g.kW * p.g.Cw) return false;
  if ((int64_t)p.M * p.lda32 * 4 > 0xffffffffLL) return false;
  if (p.g.pool && (p.N & 3)) return false;
  return true;
}

bnn_status launch_latency(GemmParams &p, int emode, int ks, hipStream_t s) {
  p.tilesM = (p.M + 31) / 32;
  p.tilesN = (p.N + 63) / 64;
  const int64_t tiles = (int64_t)p.tilesM * p.tilesN;
  if (tiles > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  ProfScope ps(KID_XNOR_CONV_LATENCY, s);
  const dim3 grid((unsigned)tiles);
  if (ks == 4) {
    if (emode == 1) hipLaunchKernelGGL((xnor_conv_latency_kernel<4, 1>), grid, dim3(1024), 0, s, p);
    else hipLaunchKernelGGL((xnor_conv_latency_kernel<4, 0>), grid, dim3(1024), 0, s, p);
  } else {
    if (emode == 1) hipLaunchKernelGGL((xnor_conv_latency_kernel<2, 1>), grid, dim3(512), 0, s, p);
    else hipLaunchKernelGGL((xnor_conv_latency_kernel<2, 0>), grid, dim3(512), 0, s, p);
  }
  return launch_status();
}

}  // namespace bnn
