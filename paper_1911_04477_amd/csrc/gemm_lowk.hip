// Xnor-Bitcount GEMM (section 3.2) for short reduction axes: rows of two or four 64-bit words
// (K <= 256), an explicit K-contiguous B, int32 / fp32 output.
//
// At such K the arithmetic is a few hundred instructions per wave and the problem is bound by
// writing the int32 / fp32 result (4 bytes out per 2 * ceil(K/32) lane-operations): what matters
// is the shape of the memory traffic, not the inner loop.
//   * a lane owns FOUR CONSECUTIVE columns, so every store is 16 bytes per lane and a wave store
//     covers 1 KB of one output row (the LDS-staged kernel, built for long rows, stores 256 B);
//   * columns that share a lane must share an image of the NCHW output: the host uses this
//     kernel only when the columns per image (and the leading dimensions) are multiples of 4,
//     which also makes every 16-byte store aligned;
//   * the whole of B a lane needs (4 rows x at most 32 bytes) is requested up front with
//     8- or 16-byte loads, no LDS, no barrier; A comes in through scalar loads, 8 rows at a
//     time, exactly as in the long-row kernel, and enters v_xor as the scalar operand;
//   * a wave computes and stores ROWS rows (one, two or four groups of 8) for its 256 columns, a
//     workgroup of four waves 4 * ROWS rows; the grid is (column tiles, row tiles);
//   * the arithmetic (a third of the store time at K = 200) only overlaps the stores if the waves
//     of a SIMD do not advance in step: workgroups get different wave priorities, and the row
//     statements carry the one-cycle yield after each pair.
// Measured on the 51.4 MB int32 output of the 1x1 / K = 200 convolution: 12.9 us (4.0 TB/s; a
// plain fill of the same buffer 9.1 us; the long-row kernel 17.9 us).
#include "common.h"
#include "gemm_rows.inc"

namespace bnn {

using u32x4 = uint32_t __attribute__((ext_vector_type(4)));
using u32x8 = uint32_t __attribute__((ext_vector_type(8)));
using i32x4 = int32_t __attribute__((ext_vector_type(4)));
using f32x4 = float __attribute__((ext_vector_type(4)));

template <int GROUPS, int HALF>  // GROUPS row groups of 8 per wave; HALF = 1: rows of two words (4 dwords)
__global__ __launch_bounds__(256) void xnor_gemm_lowk_kernel(GemmParams p) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int n = ((int)blockIdx.x * 64 + lane) * 4;  // first of this lane's four columns
  const int m_first = ((int)blockIdx.y * 4 + wave) * (8 * GROUPS);
  if (m_first >= p.M) return;  // wave-uniform; the kernel has no barrier
  const bool col_ok = n < p.N;  // N is a multiple of 4: all four columns or none
  const int nc = col_ok ? n : 0;

  // ---- B: this lane's four rows, bits past K masked, words past the row zero -------------------
  constexpr int KD = HALF ? 4 : 8;
  const int tail_bits = p.Kbits & 63;
  const uint64_t tail_mask = tail_bits ? ((1ull << tail_bits) - 1ull) : ~0ull;
  const uint32_t tm_lo = (uint32_t)tail_mask, tm_hi = (uint32_t)(tail_mask >> 32);
  uint32_t b[4][KD];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint64_t *src = p.B + (int64_t)(nc + j) * p.ldb;
    if (p.b_vec16) {
#pragma unroll
      for (int q = 0; q < KD / 4; ++q) {
        const u32x4 v = *reinterpret_cast<const u32x4 *>(src + 2 * q);
        b[j][4 * q] = v.x; b[j][4 * q + 1] = v.y; b[j][4 * q + 2] = v.z; b[j][4 * q + 3] = v.w;
      }
    } else {
#pragma unroll
      for (int w = 0; w < KD / 2; ++w) {
        const uint2 v = *reinterpret_cast<const uint2 *>(src + w);
        b[j][2 * w] = v.x; b[j][2 * w + 1] = v.y;
      }
    }
    b[j][KD - 2] &= tm_lo;
    b[j][KD - 1] &= tm_hi;
  }

  // ---- output addressing ---------------------------------------------------------------------------
  // column -> (image, pixel): row-major C is the one-image case (img_stride == 0)
  uint32_t img = 0, pix = (uint32_t)nc;
  if (p.img_stride != 0) {
    img = fdiv((uint32_t)nc, p.divOHW);
    pix = (uint32_t)nc - img * p.OHW;
  }
  const int64_t col_off = (int64_t)img * p.img_stride + pix;
  f32x4 csc = {1.f, 1.f, 1.f, 1.f}, cbi = {0.f, 0.f, 0.f, 0.f};
  if (p.Y && p.axis == BNN_CH_COL) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {  // scale / bias carry no alignment requirement
      csc[j] = p.scale[nc + j];
      cbi[j] = p.bias[nc + j];
    }
  }

  const uint32_t Abase_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)p.A);
  const uint32_t Abase_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uintptr_t)p.A >> 32));
  const uint64_t Abase = ((uint64_t)Abase_hi << 32) | (uint64_t)Abase_lo;
  const uint32_t arow_bytes = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)p.lda32 * 4u));
  const uint32_t aoff_max = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)(p.M - 1) * (uint32_t)p.lda32 * 4u));

  // Waves that share a SIMD would otherwise advance in step and all reach their stores together,
  // after the arithmetic of all of them; with different priorities they finish one after the
  // other and the stores of the first overlap the arithmetic of the rest.
  {
    const int pr = (int)((blockIdx.x + blockIdx.y) & 3u);
    if (pr == 1) __builtin_amdgcn_s_setprio(1);
    else if (pr == 2) __builtin_amdgcn_s_setprio(2);
    else if (pr == 3) __builtin_amdgcn_s_setprio(3);
  }
#pragma unroll
  for (int g = 0; g < GROUPS; ++g) {
    const int m0 = m_first + 8 * g;
    if (m0 >= p.M) break;  // wave-uniform
    // rows past M re-read row M - 1 and are not stored
    const uint32_t aoff0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)m0 * (uint32_t)p.lda32 * 4u));
    int acc[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = 0;
    uint32_t t0, t1;
#define BNN_BV(j, d) b[j][d]
    if constexpr (HALF) {
      u32x4 a[8];
#pragma unroll
      for (int i = 0; i < 8; ++i)
        asm volatile("s_load_dwordx4 %0, %1, %2" : "=s"(a[i]) : "s"(Abase), "s"(min(aoff0 + (uint32_t)i * arow_bytes, aoff_max)));
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+s"(a[0]), "+s"(a[1]), "+s"(a[2]), "+s"(a[3]), "+s"(a[4]), "+s"(a[5]), "+s"(a[6]), "+s"(a[7]));
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        a[i][2] &= tm_lo;
        a[i][3] &= tm_hi;
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) BNN_GEMM_HALF_4(acc[i], a[i], BNN_BV, t0, t1);
    } else {
      u32x8 a[8];
#pragma unroll
      for (int i = 0; i < 8; ++i)
        asm volatile("s_load_dwordx8 %0, %1, %2" : "=s"(a[i]) : "s"(Abase), "s"(min(aoff0 + (uint32_t)i * arow_bytes, aoff_max)));
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+s"(a[0]), "+s"(a[1]), "+s"(a[2]), "+s"(a[3]), "+s"(a[4]), "+s"(a[5]), "+s"(a[6]), "+s"(a[7]));
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        a[i][6] &= tm_lo;
        a[i][7] &= tm_hi;
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) BNN_GEMM_ROW_4(acc[i], a[i], BNN_BV, t0, t1);
    }
#undef BNN_BV
    // per-row affine constants of this group: wave-uniform scalar loads, requested together
    float scr[8], bir[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      scr[i] = 1.0f;
      bir[i] = 0.0f;
    }
    if (p.Y && p.axis == BNN_CH_ROW) {
      typedef const float __attribute__((address_space(4))) *cf32_ptr;
      const cf32_ptr cscale = (cf32_ptr)(uintptr_t)p.scale, cbias = (cf32_ptr)(uintptr_t)p.bias;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int mc = min(m0 + i, p.M - 1);
        scr[i] = cscale[mc];
        bir[i] = cbias[mc];
      }
    }
    if (!col_ok) continue;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int m = m0 + i;
      if (m >= p.M) break;  // wave-uniform
      i32x4 v;
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] = p.Kformula - 2 * acc[i][j];
      if (p.C) __builtin_nontemporal_store(v, reinterpret_cast<i32x4 *>(p.C + col_off + (int64_t)m * p.ldc));
      if (p.Y) {
        f32x4 y;
        if (p.axis == BNN_CH_ROW) {
#pragma unroll
          for (int j = 0; j < 4; ++j) y[j] = fmaf(scr[i], (float)v[j], bir[i]);
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j) y[j] = fmaf(csc[j], (float)v[j], cbi[j]);
        }
        __builtin_nontemporal_store(y, reinterpret_cast<f32x4 *>(p.Y + col_off + (int64_t)m * p.ldy));
      }
    }
  }
}

// Whether the short-row kernel can run the problem described by p (explicit B).
bool lowk_applicable(const GemmParams &p) {
  if (p.Kw64 != 2 && p.Kw64 != 4) return false;
  if (p.Kbits > p.Kw64 * 64 || p.Kbits <= (p.Kw64 - 1) * 64) return false;
  if ((p.N & 3) != 0) return false;
  if (p.lda32 < 2 * p.Kw64 || p.ldb < p.Kw64) return false;
  if (p.C && (p.ldc & 3)) return false;
  if (p.Y && (p.ldy & 3)) return false;
  if (p.img_stride != 0 && ((p.OHW & 3u) != 0 || (p.img_stride & 3) != 0)) return false;
  return true;
}

bnn_status launch_lowk(GemmParams &p, int groups, hipStream_t s) {
  const int64_t tilesN = ((int64_t)p.N + 255) / 256;
  const int64_t tilesM = ((int64_t)p.M + 32 * groups - 1) / (32 * groups);
  if (tilesN > 0x7fffffffLL || tilesM > 65535) return BNN_ERR_UNSUPPORTED;
  p.tilesM = (int)tilesM;
  p.tilesN = (int)tilesN;
  ProfScope ps(KID_XNOR_GEMM_LOWK, s);
  const dim3 grid((unsigned)tilesN, (unsigned)tilesM), block(256);
  const bool half = p.Kw64 == 2;
  if (groups == 4) {
    if (half) hipLaunchKernelGGL((xnor_gemm_lowk_kernel<4, 1>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((xnor_gemm_lowk_kernel<4, 0>), grid, block, 0, s, p);
  } else if (groups == 2) {
    if (half) hipLaunchKernelGGL((xnor_gemm_lowk_kernel<2, 1>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((xnor_gemm_lowk_kernel<2, 0>), grid, block, 0, s, p);
  } else {
    if (half) hipLaunchKernelGGL((xnor_gemm_lowk_kernel<1, 1>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((xnor_gemm_lowk_kernel<1, 0>), grid, block, 0, s, p);
  }
  return launch_status();
}

}  // namespace bnn
