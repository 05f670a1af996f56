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
//     are the "+1" pad word), two chunks ahead;
//   * A does NOT come through scalar loads here: with four waves per SIMD nothing hides a scalar
//     load's round trip to the L2, and it cannot be requested a chunk ahead (64 SGPRs per chunk).
//     The workgroup copies its 32 rows of A into LDS once, with one round of vector loads that
//     overlaps the first gathers, and every wave then reads its rows' chunk from LDS at one
//     address for all lanes (a broadcast, free of bank conflicts); both xor operands are vector
//     registers (last layer of the stack at batch 1: 12.7 -> 11.2 us, a whole pass 67 -> 63 us);
//   * partial counts are additive (section 3.2: a sum over the reduction axis): the slices meet
//     in LDS once, at the end, and the slice-0 waves run the epilogue -- int32 / fp32 NCHW, or
//     the binarizing epilogue (optional 2x2 max-pool, affine map, sign) that writes packed NHWC;
//   * with pooling the columns are ordered window-major with the member index in the low two
//     bits (column = 4 * window + member), so the four members of a pooling window sit in four
//     neighbouring lanes and the max is two cross-lane steps.
// Requires an even number of words per pixel (16-byte pieces never straddle a tap, rows end on a
// chunk or half-chunk boundary); the host checks it.
#include "common.h"

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

  // ---- A: the tile's 32 rows, copied to LDS once (rows past M re-read row M - 1) --------------------
  extern __shared__ __attribute__((aligned(16))) uint32_t sA[];  // [32][2 * Kw64] dwords
  {
    const int ppr = p.Kw64 >> 1;  // 16-byte pieces per row (Kw64 is even)
    const char *Ab = reinterpret_cast<const char *>(p.A);
    for (int idx = tid; idx < 32 * ppr; idx += 256 * KS) {
      const int row = idx / ppr, pc = idx - row * ppr;
      const int m = min(mi * 32 + row, p.M - 1);
      const u32x4 v = *reinterpret_cast<const u32x4 *>(Ab + (size_t)m * (size_t)p.lda32 * 4u + (size_t)pc * 16u);
      *reinterpret_cast<u32x4 *>(&sA[row * 2 * p.Kw64 + pc * 4]) = v;
    }
  }
  const uint32_t *sArow = &sA[(wm * 8) * 2 * p.Kw64];
  const int arow = 2 * p.Kw64;  // dwords per row in LDS

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
  // acc += popcount(x) as one instruction (the optimizer otherwise splits it into a popcount and an add)
  auto popc_acc = [](uint32_t x, int a) {
    asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(a) : "v"(x));
    return a;
  };
  auto compute = [&](const u32x8 &bv, int cl) {
    const uint32_t *ac = sArow + (cb + cl) * 8;
    // two rows of A in flight at a time: more would not fit the 128 registers a 1024-thread workgroup leaves a lane
#pragma unroll
    for (int i = 0; i < 8; i += 2) {
      const u32x4 a0 = *reinterpret_cast<const u32x4 *>(ac + i * arow);
      const u32x4 a1 = *reinterpret_cast<const u32x4 *>(ac + i * arow + 4);
      const u32x4 c0 = *reinterpret_cast<const u32x4 *>(ac + (i + 1) * arow);
      const u32x4 c1 = *reinterpret_cast<const u32x4 *>(ac + (i + 1) * arow + 4);
      int t = acc[i][0], u = acc[i + 1][0];
#pragma unroll
      for (int d = 0; d < 4; ++d) t = popc_acc(a0[d] ^ bv[d], t);
#pragma unroll
      for (int d = 0; d < 4; ++d) t = popc_acc(a1[d] ^ bv[4 + d], t);
#pragma unroll
      for (int d = 0; d < 4; ++d) u = popc_acc(c0[d] ^ bv[d], u);
#pragma unroll
      for (int d = 0; d < 4; ++d) u = popc_acc(c1[d] ^ bv[4 + d], u);
      acc[i][0] = t;
      acc[i + 1][0] = u;
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  u32x8 bq[DEPTH];
#pragma unroll
  for (int d = 0; d < DEPTH; ++d)
    if (d < nfull) load_b(bq[d], d);
  __syncthreads();  // the copy of A is complete (its loads and the first gathers were in flight together)
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
    const uint32_t *ac = sArow + nfull_all * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const u32x4 a0 = *reinterpret_cast<const u32x4 *>(ac + i * arow);
      int t = acc[i][0];
#pragma unroll
      for (int d = 0; d < 4; ++d) t = popc_acc(a0[d] ^ bv[d], t);
      acc[i][0] = t;
    }
  }

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
      typedef const float __attribute__((address_space(4))) *cf32_ptr;
      const cf32_ptr cscale = (cf32_ptr)(uintptr_t)p.scale, cbias = (cf32_ptr)(uintptr_t)p.bias;
      float scr[8], bir[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        scr[i] = 1.0f;
        bir[i] = 0.0f;
      }
      if (p.Y) {  // wave-uniform scalar loads, requested together; rows past M re-read row M - 1
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int mc = min(m0 + i, p.M - 1);
          scr[i] = cscale[mc];
          bir[i] = cbias[mc];
        }
      }
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
            if (p.Y) p.Y[off + (int64_t)m * p.ldy] = fmaf(scr[i], (float)v, bir[i]);
          }
        }
      }
    } else {
      // binarizing epilogue: K - 2*acc decreases in acc, so the 2x2 max is K - 2*min(acc) over the
      // four neighbouring lanes of a window; rows run from the last to the first so that each sign
      // is shifted in with one add
      // the 8 rows' affine constants: wave-uniform scalar loads, requested together
      typedef const float __attribute__((address_space(4))) *cf32_ptr;
      const cf32_ptr cscale = (cf32_ptr)(uintptr_t)p.scale, cbias = (cf32_ptr)(uintptr_t)p.bias;
      float scr[8], bir[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int mc = min(m0 + i, p.M - 1);
        scr[i] = cscale[mc];
        bir[i] = cbias[mc];
      }
      uint32_t byte = 0u;
#pragma unroll
      for (int i = 7; i >= 0; --i) {
        const int m = m0 + i;
        const bool row_ok = m < p.M;
        const float sc = row_ok ? scr[i] : 0.0f;
        const float bi = row_ok ? bir[i] : -1.0f;  // rows past M give bit 0
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
  if (p.lda32 != 2 * p.Kw64) return false;                    // rows of A contiguous: 16-byte aligned row starts
  if ((int64_t)32 * p.Kw64 * 8 > 24 * 1024) return false;     // the tile's rows of A must fit the LDS left beside the partial sums
  return true;
}

bnn_status launch_latency(GemmParams &p, int emode, int ks, hipStream_t s) {
  p.tilesM = (p.M + 31) / 32;
  p.tilesN = (p.N + 63) / 64;
  const int64_t tiles = (int64_t)p.tilesM * p.tilesN;
  if (tiles > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  ProfScope ps(KID_XNOR_CONV_LATENCY, s);
  const dim3 grid((unsigned)tiles);
  const size_t lds = (size_t)32 * p.Kw64 * 8;  // the tile's rows of A
  if (ks == 4) {
    if (emode == 1) hipLaunchKernelGGL((xnor_conv_latency_kernel<4, 1>), grid, dim3(1024), lds, s, p);
    else hipLaunchKernelGGL((xnor_conv_latency_kernel<4, 0>), grid, dim3(1024), lds, s, p);
  } else {
    if (emode == 1) hipLaunchKernelGGL((xnor_conv_latency_kernel<2, 1>), grid, dim3(512), lds, s, p);
    else hipLaunchKernelGGL((xnor_conv_latency_kernel<2, 0>), grid, dim3(512), lds, s, p);
  }
  return launch_status();
}

}  // namespace bnn
