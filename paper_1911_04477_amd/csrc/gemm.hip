// Xnor-Bitcount GEMM (section 3.2 of the paper) for gfx950, in the exclusive-or form
//     C[m,n] = K - 2 * sum_w popcount(A[m,w] ^ B[n,w]).
//
// CDNA4 has no 1-bit matrix instruction, so the contraction runs on the vector ALU:
// two lane-instructions per 32 bit-MACs per output (v_xor_b32, then v_bcnt_u32_b32
// which adds its popcount into the accumulator).  The kernel is built so that the
// inner loop is almost nothing else:
//   * lanes of a wave run along N (64 consecutive columns per register column);
//     every lane keeps 8 x TN int32 accumulators;
//   * the 8 rows of A a wave works on are the same for all of its lanes, so A is
//     fetched with SCALAR loads into SGPRs and enters v_xor as the scalar operand:
//     no LDS traffic, no VGPRs and no VALU instructions are spent on A;
//   * the block's B tile (BN columns x 8 dwords) is staged once per K-chunk through
//     double-buffered LDS, row-per-column with a 4-dword pad so that both the 16-byte
//     staging writes and the 16-byte per-lane reads are bank-conflict free; the next
//     chunk's global loads are issued before the current chunk is computed and first
//     touched after it;
//   * B is either an explicit K-contiguous matrix or (implicit GEMM) gathered on the
//     fly from a packed NHWC image: column = output pixel, row word = tap word, pad
//     taps replaced by the "+1" word -- no patch matrix is ever written.  The gather has
//     a general form (BMODE 1) and a lean one (BMODE 2) that keeps every division and all
//     geometry out of the chunk loop: a per-slot tap-validity mask and 32-bit base offset,
//     and a per-workgroup LDS table of tap offsets;
//   * K tails: two leftover words run a half chunk; one or three re-read the final 8
//     dwords of the rows (a window that overlaps the previous chunk) with the overlap and
//     the bits past K zeroed in both operands (A in SGPRs with scalar moves, B in the
//     staging), so they run the same instruction sequence as a full chunk; rows shorter
//     than four words go one dword at a time;
//   * everything a chunk needs besides the math is kept off the vector ALU and out of
//     long-lived SGPRs (row offsets are recomputed by scalar adds per chunk), because the
//     kernel is VALU-bound and SGPR spills are VALU instructions (v_readlane);
//   * the store does K - 2*acc and then either writes int32 / fma(scale, acc, bias) fp32
//     (row-major or scattered to NCHW; 256 contiguous bytes per wave store, or, on the
//     256-column tiles when N and the strides are multiples of 4, 1 KB: the tile's columns are
//     then dealt to the LDS rows so that a lane's four columns are consecutive), or -- the
//     binarizing epilogue -- takes the 2x2 max (optional), applies the fma, keeps only the
//     sign and writes packed NHWC words for the next layer (32x fewer output bytes).
// Workgroup ids are remapped so that tiles sharing a B tile run on the same XCD
// (one L2 per XCD; hardware deals consecutive ids round-robin over the 8 XCDs).
#include "common.h"
#include "bnn_testing.h"
#include "gemm_rows.inc"

namespace bnn {

using u32x4 = uint32_t __attribute__((ext_vector_type(4)));
using u32x8 = uint32_t __attribute__((ext_vector_type(8)));
// A is only ever read by the kernel.  Reading it through the constant address space lets
// the compiler use scalar (SMEM) loads for wave-uniform addresses.
#define BNN_CONST_AS __attribute__((address_space(4)))
typedef const uint32_t BNN_CONST_AS *cu32_ptr;

// acc += popcount(x) as ONE instruction.  Written as asm because the optimizer otherwise
// re-associates a chain of popcount-adds into v_bcnt(x, 0) plus separate three-operand adds.
__device__ __forceinline__ int popc_acc(uint32_t x, int acc) {
  asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc) : "v"(x));
  return acc;
}

// The K axis is consumed in chunks of KC = 8 dwords (256 bits); a wave owns TM = 8 rows.
constexpr int KC = 8;
constexpr int TM = 8;
// lean implicit gather: chunks per row the per-workgroup tap table holds, and its flag bits
constexpr int LEAN_MAX_STAGES = 512;
constexpr uint32_t LEAN_LIVE = 1u, LEAN_TAP_END = 2u;

template <int TN, int WM, int WN>
struct GemmCfg {
  static constexpr int BM = TM * WM;
  static constexpr int BN = 64 * TN * WN;
  static constexpr int THREADS = 64 * WM * WN;
  static constexpr int RS = KC + 4;                      // LDS row stride in dwords
  static constexpr int TILE = BN * RS;                   // dwords per LDS buffer
  static constexpr int PIECES = BN * (KC / 4);           // 16-byte pieces per chunk
  static constexpr int PPT = (PIECES + THREADS - 1) / THREADS;
  static_assert(PIECES % THREADS == 0 || PIECES < THREADS, "staging must divide evenly");
};

// words of a tap that lies outside the image: every real channel is +1 (bit 1)
__device__ __forceinline__ uint64_t pad_word64(int C, int cw) {
  const int left = C - cw * 64;
  return left >= 64 ? ~0ull : (left <= 0 ? 0ull : ((1ull << left) - 1ull));
}

// Column n of an implicit GEMM -> output pixel.  Without pooling the columns are the
// output pixels in NHWC order.  With 2x2 pooling a tile of 256 columns holds 64 pooling
// windows: column 256*t + 64*j + l is member j (row-major in the 2x2 window) of window
// 64*t + l, so that the four members of a window are the four register columns of one lane.
__device__ __forceinline__ void decode_col(const ConvGeom &g, uint32_t n, uint32_t &img, int &oh, int &ow) {
  if (g.pool == 0) {
    const uint32_t t = fdiv(n, g.divOW);
    ow = (int)(n - t * g.OW);
    img = fdiv(t, g.divOH);
    oh = (int)(t - img * g.OH);
  } else {
    const uint32_t j = (n >> 6) & 3u;
    const uint32_t wdx = (n >> 8) * 64u + (n & 63u);
    const uint32_t PW = g.OW >> 1, PH = g.OH >> 1;
    const uint32_t t = fdiv(wdx, g.divOW);
    const uint32_t wx = wdx - t * PW;
    img = fdiv(t, g.divOH);
    const uint32_t wy = t - img * PH;
    oh = (int)(2 * wy + (j >> 1));
    ow = (int)(2 * wx + (j & 1));
  }
}

// Store of an 8 x TN accumulator tile: K - 2*acc as int32 and / or fma(scale, acc, bias) as
// fp32, row-major or scattered to NCHW.  The store-only parameters are read from the
// kernel-argument segment through a pointer the optimizer cannot see through, so that they
// occupy no SGPRs (or spill slots) during the main loop.
template <int TN>
__device__ __forceinline__ void store_tile(const int (&acc)[TM][TN], int m0, int nbase) {
  const GemmParams BNN_CONST_AS *kp = (const GemmParams BNN_CONST_AS *)__builtin_amdgcn_kernarg_segment_ptr();
  asm volatile("" : "+s"(kp));
  const int M = kp->M, N = kp->N, Kformula = kp->Kformula;
  const float *const scale = kp->scale, *const bias = kp->bias;
  const int axis = kp->axis;
  int32_t *const Cp = kp->C;
  float *const Yp = kp->Y;
  const int64_t ldc = kp->ldc, ldy = kp->ldy, img_stride = kp->img_stride;
  const uint32_t OHW = kp->OHW;
  // Non-temporal stores when every 256-byte piece a wave stores covers whole 128-byte lines (measured
  // 1 % faster then); ordinary stores otherwise, so that pieces that share a line meet in the L2
  // instead of each going to memory as a partial line (49.6 -> 40.7 us on a 31 x 33 map).
  const bool nt = kp->nt_store != 0;
  FastDiv divOHW;
  divOHW.d = kp->divOHW.d; divOHW.mul = kp->divOHW.mul; divOHW.shift = kp->divOHW.shift;
  // per-row affine constants once per tile (wave-uniform: scalar loads; rows past M re-read row M - 1)
  typedef const float BNN_CONST_AS *cf32_ptr;
  const cf32_ptr cscale = (cf32_ptr)(uintptr_t)scale, cbias = (cf32_ptr)(uintptr_t)bias;
  float scr[TM], bir[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    scr[i] = 1.0f;
    bir[i] = 0.0f;
  }
  if (Yp && axis == BNN_CH_ROW) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int mi = min(m0 + i, M - 1);
      scr[i] = cscale[mi];
      bir[i] = cbias[mi];
    }
  }
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int n = nbase + j * 64;
    if (n >= N) continue;
    const uint32_t img = fdiv((uint32_t)n, divOHW);
    const uint32_t pix = (uint32_t)n - img * OHW;
    const int64_t coff = (int64_t)img * img_stride + pix + (int64_t)m0 * ldc;
    const int64_t yoff = (int64_t)img * img_stride + pix + (int64_t)m0 * ldy;
    int32_t *cp = Cp ? Cp + coff : nullptr;
    float *yp = Yp ? Yp + yoff : nullptr;
    float sc = 1.0f, bi = 0.0f;
    if (Yp && axis == BNN_CH_COL) {
      sc = scale[n];
      bi = bias[n];
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      if (m0 + i < M) {
        const int v = Kformula - 2 * acc[i][j];
        if (cp) {
          if (nt) __builtin_nontemporal_store(v, cp);
          else *cp = v;
        }
        if (yp) {
          const float s1 = axis == BNN_CH_ROW ? scr[i] : sc, b1 = axis == BNN_CH_ROW ? bir[i] : bi;
          const float y = fmaf(s1, (float)v, b1);
          if (nt) __builtin_nontemporal_store(y, yp);
          else *yp = y;
        }
      }
      if (cp) cp += ldc;
      if (yp) yp += ldy;
    }
  }
}

// The same store for a column-permuted tile (GemmParams::colperm): the lane's four accumulators of a
// row are four consecutive columns, first column nfirst (a multiple of 4), stored with one 16-byte
// store per row.  The host sets colperm only where N, the leading dimensions and the columns per
// image are multiples of 4, so the four columns are all inside or all outside the matrix, lie in one
// image and start on a 16-byte boundary.
__device__ __forceinline__ void store_tile_x4(const int (&acc)[TM][4], int m0, int nfirst) {
  using i32x4 = int __attribute__((ext_vector_type(4)));
  using f32x4 = float __attribute__((ext_vector_type(4)));
  const GemmParams BNN_CONST_AS *kp = (const GemmParams BNN_CONST_AS *)__builtin_amdgcn_kernarg_segment_ptr();
  asm volatile("" : "+s"(kp));
  const int M = kp->M, N = kp->N, Kformula = kp->Kformula;
  if (nfirst >= N) return;
  const float *const scale = kp->scale, *const bias = kp->bias;
  const int axis = kp->axis;
  int32_t *const Cp = kp->C;
  float *const Yp = kp->Y;
  const int64_t ldc = kp->ldc, ldy = kp->ldy, img_stride = kp->img_stride;
  const uint32_t OHW = kp->OHW;
  const bool nt = kp->nt_store != 0;
  FastDiv divOHW;
  divOHW.d = kp->divOHW.d; divOHW.mul = kp->divOHW.mul; divOHW.shift = kp->divOHW.shift;
  typedef const float BNN_CONST_AS *cf32_ptr;
  const cf32_ptr cscale = (cf32_ptr)(uintptr_t)scale, cbias = (cf32_ptr)(uintptr_t)bias;
  float scr[TM], bir[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    scr[i] = 1.0f;
    bir[i] = 0.0f;
  }
  if (Yp && axis == BNN_CH_ROW) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int mi = min(m0 + i, M - 1);
      scr[i] = cscale[mi];
      bir[i] = cbias[mi];
    }
  }
  f32x4 csc = {1.f, 1.f, 1.f, 1.f}, cbi = {0.f, 0.f, 0.f, 0.f};
  if (Yp && axis == BNN_CH_COL) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {  // scale / bias carry no alignment requirement
      csc[j] = scale[nfirst + j];
      cbi[j] = bias[nfirst + j];
    }
  }
  const uint32_t img = fdiv((uint32_t)nfirst, divOHW);
  const uint32_t pix = (uint32_t)nfirst - img * OHW;
  int32_t *cp = Cp ? Cp + ((int64_t)img * img_stride + pix + (int64_t)m0 * ldc) : nullptr;
  float *yp = Yp ? Yp + ((int64_t)img * img_stride + pix + (int64_t)m0 * ldy) : nullptr;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    if (m0 + i < M) {
      i32x4 v;
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] = Kformula - 2 * acc[i][j];
      if (cp) {
        if (nt) __builtin_nontemporal_store(v, reinterpret_cast<i32x4 *>(cp));
        else *reinterpret_cast<i32x4 *>(cp) = v;
      }
      if (yp) {
        f32x4 y;
#pragma unroll
        for (int j = 0; j < 4; ++j)
          y[j] = axis == BNN_CH_ROW ? fmaf(scr[i], (float)v[j], bir[i]) : fmaf(csc[j], (float)v[j], cbi[j]);
        if (nt) __builtin_nontemporal_store(y, reinterpret_cast<f32x4 *>(yp));
        else *reinterpret_cast<f32x4 *>(yp) = y;
      }
    }
    if (cp) cp += ldc;
    if (yp) yp += ldy;
  }
}

template <int TN, int WM, int WN, int MINW, int BMODE, int EMODE, int YIELD>
__global__ __launch_bounds__(64 * WM * WN, MINW) void xnor_gemm_kernel(GemmParams p) {
  using Cfg = GemmCfg<TN, WM, WN>;
  constexpr int RS = Cfg::RS;
  constexpr int PPT = Cfg::PPT;
  constexpr int QPR = KC / 4;  // 16-byte pieces per row
  static_assert(EMODE == 0 || ((WM == 8 || WM == 4) && WN == 1 && (TN == 4 || TN == 2)),
                "packed epilogue needs 64- or 32-row tiles");
  __shared__ __attribute__((aligned(16))) uint32_t sB[2 * Cfg::TILE];
  __shared__ uint2 sTab[BMODE == 2 ? 2 * LEAN_MAX_STAGES : 1];

  __builtin_amdgcn_s_setprio(3);  // prologue and epilogue are short and latency-bound: let them through
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % WM;
  const int wn = wave / WM;

  // XCD-aware tile order: ids that land on one XCD get consecutive tiles.
  const uint32_t nb = gridDim.x, bid = blockIdx.x;
  const uint32_t xcd = bid & 7u, loc = bid >> 3;
  const uint32_t base = nb >> 3, rem = nb & 7u;
  const uint32_t tile = xcd * base + (xcd < rem ? xcd : rem) + loc;
  const int mi = (int)(tile % (uint32_t)p.tilesM);
  const int ni = (int)(tile / (uint32_t)p.tilesM);
  const int m0 = mi * Cfg::BM + wm * TM;
  const int n0 = ni * Cfg::BN;
  // Tile column held by LDS row `row` of the B tile: the row itself, or (column-permuted tiles, see
  // GemmParams::colperm) 4 * (row % 64) + row / 64.
  const bool colperm = EMODE == 0 && TN == 4 && WN == 1 && p.colperm != 0;
  auto tile_col = [&](int row) { return colperm ? ((row & 63) << 2) + (row >> 6) : row; };

  // Byte offsets of this wave's TM rows: first row + i * row bytes, clamped to the last row of A
  // (rows past M recompute row M-1 and are not stored).  Three SGPRs; the eight offsets are
  // recomputed on the scalar unit every chunk instead of living in (spilled) registers.
  // 32-bit: the host checks that M * lda32 * 4 < 2^32.
  const uint32_t arow_bytes = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)p.lda32 * 4u));
  const uint32_t aoff_max = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)(p.M - 1) * (uint32_t)p.lda32 * 4u));
  uint32_t aoff_first;
  {
    const int mf = m0 < p.M ? m0 : p.M - 1;
    aoff_first = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)mf * (uint32_t)p.lda32 * 4u));
  }
  // Re-defining the first offset through an empty asm inside the loop keeps the compiler from
  // hoisting the eight derived offsets out of it.
#define BNN_AOFF(i) min(aoff_cur + (uint32_t)(i) * arow_bytes, aoff_max)
  // 64-bit base of A in an SGPR pair (readfirstlane returns a signed int: each half is cast
  // to unsigned before widening).
  const uint32_t Abase_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)p.A);
  const uint32_t Abase_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uintptr_t)p.A >> 32));
  const uint64_t Abase0 = ((uint64_t)Abase_hi << 32) | (uint64_t)Abase_lo;
  const cu32_ptr Ac = (cu32_ptr)(uintptr_t)p.A;

  // Zeroed through an opaque statement: a plain "= 0" is re-materialised by the compiler on
  // every path into the loop (the accumulators were cleared twice per tile).
  int acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) asm volatile("v_mov_b32 %0, 0" : "=v"(acc[i][j]));

  // K bookkeeping (all wave-uniform).  Full chunks cover words [0, 4*nfull).  Two words left
  // over are done by a half chunk; one or three by a last "window" chunk over words
  // [Kw64-4, Kw64) when the row has at least 4 words; else one dword at a time.
  const int nfull = p.Kbits / (32 * KC);
  const int rem_bits = p.Kbits - nfull * 32 * KC;
  const int r_words = p.Kw64 - 4 * nfull;                           // words past the full chunks: 0..3
  const bool half = r_words == 2;                                   // finished by one half chunk (4 dwords)
  const bool window = BMODE != 2 && rem_bits > 0 && !half && p.Kw64 >= 4;  // finished by an overlapping chunk
  const bool slow_tail = BMODE != 2 && rem_bits > 0 && !half && !window;   // rows of 1 or 3 words only
  const int nstages = nfull + (rem_bits > 0 ? 1 : 0);
  const int last_w = p.Kw64 - 1;
  const int tail_bits = p.Kbits & 63;
  const uint64_t tail_mask = tail_bits ? ((1ull << tail_bits) - 1ull) : ~0ull;
  // first word of stage s: 4*s for full chunks (and for the slow tail), Kw64-4 for the window
  auto stage_word0 = [&](int s) { return (s == nfull && window) ? p.Kw64 - 4 : 4 * s; };

  // ---- staging: global -> registers -> LDS (double-buffered) -----------------------
  // Per-slot constants of the implicit-GEMM gather (one output pixel per slot).
  int s_ih0[PPT], s_iw0[PPT];
  uint32_t s_pix0[PPT];
  bool s_ok[PPT];
  if constexpr (BMODE == 1) {
#pragma unroll
    for (int t = 0; t < PPT; ++t) {
      const int idx = t * Cfg::THREADS + tid;
      const int row = idx / QPR;
      const uint32_t n = (uint32_t)(n0 + tile_col(row));
      // pooled ordering: a column is real iff its window exists (N = 4 * windows, but the
      // columns of the last tile's missing windows are interleaved with real ones)
      const uint32_t wdx = (n >> 8) * 64u + (n & 63u);
      s_ok[t] = idx < Cfg::PIECES && (p.g.pool ? wdx < (uint32_t)(p.N >> 2) : n < (uint32_t)p.N);
      uint32_t img = 0;
      int oh = 0, ow = 0;
      if (s_ok[t]) decode_col(p.g, n, img, oh, ow);
      s_ih0[t] = oh * p.g.sH - p.g.pH;
      s_iw0[t] = ow * p.g.sW - p.g.pW;
      s_pix0[t] = img * (uint32_t)(p.g.H * p.g.W);
    }
  }
  // Lean gather (BMODE 2: even Cw, at most 32 taps, image under 4 GiB, at most LEAN_MAX_STAGES
  // chunks).  Per slot: the byte offset of the pixel under tap (0, 0) (may be "negative": 32-bit
  // wrap-around arithmetic, only used for taps inside the image) and one validity bit per tap.
  // Per (chunk, 16-byte piece): an LDS table entry {byte offset of the tap word | flags, tap bit},
  // built once per workgroup, so the loop holds no division, no geometry and no scalar state for
  // the gather: a chunk costs a lane one LDS read, one and, one compare, one add, one select.
  uint32_t f_base[PPT], f_vmask[PPT];
  bool f_valid[PPT];
  const int my_piece = tid & 1;  // a thread always stages the same piece of a chunk
  if constexpr (BMODE == 2) {
    static_assert(QPR == 2, "two pieces per chunk");
#pragma unroll
    for (int t = 0; t < PPT; ++t) {
      const int idx = t * Cfg::THREADS + tid;
      const int row = idx / QPR;
      const uint32_t n = (uint32_t)(n0 + tile_col(row));
      const uint32_t wdx = (n >> 8) * 64u + (n & 63u);
      const bool ok = idx < Cfg::PIECES && (p.g.pool ? wdx < (uint32_t)(p.N >> 2) : n < (uint32_t)p.N);
      uint32_t img = 0;
      int oh = 0, ow = 0;
      if (ok) decode_col(p.g, n, img, oh, ow);
      const int ih0 = oh * p.g.sH - p.g.pH, iw0 = ow * p.g.sW - p.g.pW;
      uint32_t colbits = 0, vm = 0;
#pragma unroll 1
      for (int kw = 0; kw < p.g.kW; ++kw) colbits |= (uint32_t)(iw0 + kw >= 0 && iw0 + kw < p.g.W) << kw;
#pragma unroll 1
      for (int kh = 0; kh < p.g.kH; ++kh)
        if (ih0 + kh >= 0 && ih0 + kh < p.g.H) vm |= colbits << (kh * p.g.kW);
      f_vmask[t] = ok ? vm : 0u;  // columns past N read nothing but pad words and are not stored
      f_base[t] = (uint32_t)((((int64_t)img * p.g.H + ih0) * p.g.W + iw0) * p.g.Cw * 8);
      f_valid[t] = false;
    }
    // entry e = 2 * chunk + piece: words w = 2 e, 2 e + 1 of the row (same tap: Cw is even)
    const int n_entries = 2 * nstages;
    for (int e = tid; e < n_entries; e += Cfg::THREADS) {
      const uint32_t w = 2u * (uint32_t)e;
      const uint32_t tap = fdiv(w, p.g.divCw);
      const uint32_t cw = w - tap * (uint32_t)p.g.Cw;
      const uint32_t kh = fdiv(tap, p.g.divKW);
      const uint32_t kw = tap - kh * (uint32_t)p.g.kW;
      const bool live = (int)w <= last_w;  // words past K: no tap, pad word 0
      uint32_t lo = ((kh * (uint32_t)p.g.W + kw) * (uint32_t)p.g.Cw + cw) * 8u;  // multiple of 16
      if (live) lo |= LEAN_LIVE;
      if ((int)cw + 2 == p.g.Cw) lo |= LEAN_TAP_END;
      sTab[e] = make_uint2(lo, live ? (1u << tap) : 0u);
    }
    __syncthreads();
  }
  // One word of an implicit B row: tap = w / Cw, channel word = w % Cw.
  auto gather_word = [&](int t, int w) -> uint64_t {
    const uint32_t tap = fdiv((uint32_t)w, p.g.divCw);
    const int cw = w - (int)tap * p.g.Cw;
    const uint32_t kh = fdiv(tap, p.g.divKW);
    const int kw = (int)(tap - kh * p.g.kW);
    const int ih = s_ih0[t] + (int)kh, iw = s_iw0[t] + kw;
    if (ih >= 0 && ih < p.g.H && iw >= 0 && iw < p.g.W)
      return p.g.act[((size_t)s_pix0[t] + (size_t)(ih * p.g.W + iw)) * p.g.Cw + cw];
    return pad_word64(p.g.C, cw);
  };

  // stage_load only ISSUES the global loads (raw words stay in registers, nothing uses them
  // until stage_store a whole chunk of compute later), so their latency is never waited on.
  u32x4 stage[PPT];
  uint32_t staged_flags = 0;  // lean gather: flags of the table entry the last stage_load used
  auto stage_load = [&](int s) {
    const int wbase = stage_word0(s);
    if constexpr (BMODE == 2) {
      // (both words are used unconditionally, the flags by stage_store: one 8-byte LDS read; when
      // only the offset depended on it the compiler fetched it behind a branch, for valid taps only)
      const uint2 ent = sTab[2 * s + my_piece];
      staged_flags = ent.x;  // stage_store(s) selects the pad word by the same entry
      const uint32_t my_off = ent.x & ~15u;
      const char *base = reinterpret_cast<const char *>(p.g.act);
#pragma unroll
      for (int t = 0; t < PPT; ++t) {
        const bool valid = (f_vmask[t] & ent.y) != 0u;
        const uint32_t off = valid ? f_base[t] + my_off : 0u;  // taps outside: any readable address
        f_valid[t] = valid;
        stage[t] = *reinterpret_cast<const u32x4 *>(base + off);
      }
      return;
    }
    int tap_cw[2] = {0, 0}, tap_kh[2] = {0, 0}, tap_kw[2] = {0, 0};
    if constexpr (BMODE == 1) {
#pragma unroll
      for (int qq = 0; qq < 2; ++qq) {
        const uint32_t w = (uint32_t)__builtin_amdgcn_readfirstlane(wbase + 2 * qq);
        const uint32_t tap = fdiv(w, p.g.divCw);
        tap_cw[qq] = (int)(w - tap * (uint32_t)p.g.Cw);
        const uint32_t kh = fdiv(tap, p.g.divKW);
        tap_kh[qq] = (int)kh;
        tap_kw[qq] = (int)(tap - kh * (uint32_t)p.g.kW);
      }
    }
#pragma unroll
    for (int t = 0; t < PPT; ++t) {
      const int idx = t * Cfg::THREADS + tid;
      const int row = idx / QPR, q = idx % QPR;
      const int w0 = wbase + 2 * q;
      u32x4 v = {0u, 0u, 0u, 0u};
      if constexpr (BMODE == 0) {
        const int n = n0 + tile_col(row);
        if (idx < Cfg::PIECES && n < p.N && w0 <= last_w) {
          const uint64_t *src = p.B + (int64_t)n * p.ldb + w0;
          if (p.b_vec16 && !(wbase & 1) && w0 + 1 <= last_w) {
            v = *reinterpret_cast<const u32x4 *>(src);
          } else {
            const uint2 lo = *reinterpret_cast<const uint2 *>(src);
            v.x = lo.x; v.y = lo.y;
            if (w0 + 1 <= last_w) {
              const uint2 hi = *reinterpret_cast<const uint2 *>(src + 1);
              v.z = hi.x; v.w = hi.y;
            }
          }
        }
      } else {
        if (s_ok[t] && w0 <= last_w) {
          if (!(p.g.Cw & 1) && !(wbase & 1)) {
            // both words of the piece belong to one tap: one 16-byte load.  The tap of each of
            // the two pieces of a chunk is wave-uniform (decoded once per chunk on the scalar
            // unit, see tap_* below); a lane only selects by its piece index q.
            const int cw = q ? tap_cw[1] : tap_cw[0];
            const int ih = s_ih0[t] + (q ? tap_kh[1] : tap_kh[0]);
            const int iw = s_iw0[t] + (q ? tap_kw[1] : tap_kw[0]);
            if (ih >= 0 && ih < p.g.H && iw >= 0 && iw < p.g.W) {
              v = *reinterpret_cast<const u32x4 *>(
                  p.g.act + ((size_t)s_pix0[t] + (size_t)(ih * p.g.W + iw)) * p.g.Cw + cw);
            } else {
              const uint64_t x0 = pad_word64(p.g.C, cw), x1 = pad_word64(p.g.C, cw + 1);
              v.x = (uint32_t)x0; v.y = (uint32_t)(x0 >> 32); v.z = (uint32_t)x1; v.w = (uint32_t)(x1 >> 32);
            }
          } else {
            const uint64_t x0 = gather_word(t, w0);
            const uint64_t x1 = w0 + 1 <= last_w ? gather_word(t, w0 + 1) : 0ull;
            v.x = (uint32_t)x0; v.y = (uint32_t)(x0 >> 32); v.z = (uint32_t)x1; v.w = (uint32_t)(x1 >> 32);
          }
        }
      }
      stage[t] = v;
    }
  };
  // Zeroes the words a window chunk shares with the full chunks before it, masks the bits
  // past K in the row's last word, then writes the pieces to LDS buffer buf.
  auto stage_store = [&](int buf, int s) {
    const int wbase = stage_word0(s);
    if constexpr (BMODE == 2) {
      // pad words: all ones, except the last word of a tap (low C % 64 bits) and words past K (0);
      // rows hold whole words, so there is no tail mask
      const uint32_t fl = staged_flags;
      const uint64_t last = pad_word64(p.g.C, p.g.Cw - 1);
      const uint32_t a1 = (fl & LEAN_LIVE) ? 0xffffffffu : 0u;
      const bool te = (fl & LEAN_TAP_END) != 0u;
      const u32x4 padv = {a1, a1, te ? (uint32_t)last & a1 : a1, te ? (uint32_t)(last >> 32) & a1 : a1};
#pragma unroll
      for (int t = 0; t < PPT; ++t) {
        const int idx = t * Cfg::THREADS + tid;
        const int row = idx / QPR, q = idx % QPR;
        const u32x4 v = f_valid[t] ? stage[t] : padv;
        if (idx < Cfg::PIECES) *reinterpret_cast<u32x4 *>(&sB[buf * Cfg::TILE + row * RS + q * 4]) = v;
      }
      return;
    }
    const int wdone = (s == nfull && window) ? 4 * nfull : 0;  // words below this are already counted
    const uint32_t tm_lo = (uint32_t)tail_mask, tm_hi = (uint32_t)(tail_mask >> 32);
#pragma unroll
    for (int t = 0; t < PPT; ++t) {
      const int idx = t * Cfg::THREADS + tid;
      const int row = idx / QPR, q = idx % QPR;
      const int w0 = wbase + 2 * q;
      u32x4 v = stage[t];
      if (w0 == last_w) { v.x &= tm_lo; v.y &= tm_hi; }
      if (w0 + 1 == last_w) { v.z &= tm_lo; v.w &= tm_hi; }
      if (w0 < wdone) { v.x = 0u; v.y = 0u; }
      if (w0 + 1 < wdone) { v.z = 0u; v.w = 0u; }
      if (idx < Cfg::PIECES) *reinterpret_cast<u32x4 *>(&sB[buf * Cfg::TILE + row * RS + q * 4]) = v;
    }
  };

  const int lane_row = (wn * 64 * TN + lane) * RS;

  if (nstages > 0) {
    stage_load(0);
    stage_store(0, 0);
  }
  __syncthreads();

  // ---- chunks ----------------------------------------------------------------------------
  // Per chunk: the wave's 8 rows of A arrive with 8 scalar loads of 8 dwords (64 SGPRs),
  // issued together with the LDS reads of B; one wait; then 2 * 8 * TN * 8 xor / popcount
  // instructions and nothing else.  Loads, wait and the per-row compute statements are
  // volatile inline asm, so their order in the instruction stream is the order written
  // here; the wait names every loaded SGPR as in/out operand, which orders all uses after
  // it.  The latency of one wave's loads is covered by the other waves on the SIMD.
  const int nfast = nfull + (window ? 1 : 0);
  // Wave priority.  The instruction arbiter prefers older waves, so of the workgroups resident
  // on a compute unit the oldest runs at nearly full speed, the others in its gaps, and they
  // finish one after the other; the last one then runs alone, at an occupancy where neither its
  // latencies nor the yield slots of its pairs are filled.  The workgroups of the last resident
  // set (ids >= prio_from) therefore lower their priority as they advance through K: whoever is
  // behind gets the issue slots, and they finish within an eighth of K of each other.  Earlier
  // workgroups keep one priority and free their slot as early as before.
  const bool paced = (int)blockIdx.x >= p.prio_from;
  // Prologue and store run at priority 3 (set at kernel entry and before the store): they are
  // short and latency-bound, and a new workgroup that gets through its prologue quickly is one
  // more set of waves with work to issue.  The K loop runs below that: at 2 for the earlier
  // workgroups, stepping down from 2 for the paced ones (from 3 when every workgroup of the
  // launch is paced, so that the steps at 1/2, 3/4 and 7/8 of K all exist).
  const int prio_top = p.prio_from == 0 ? 3 : 2;
  int prio_cur = prio_top;
  if (prio_top == 2) __builtin_amdgcn_s_setprio(2);
  for (int c = 0; c < nfast; ++c) {
    if (paced) {
      const int steps = (2 * c < nstages) ? 0 : (4 * c < 3 * nstages) ? 1 : (8 * c < 7 * nstages) ? 2 : 3;
      const int lvl = max(prio_top - steps, 0);  // wave-uniform
      if (lvl != prio_cur) {
        prio_cur = lvl;
        if (lvl == 2) __builtin_amdgcn_s_setprio(2);
        else if (lvl == 1) __builtin_amdgcn_s_setprio(1);
        else __builtin_amdgcn_s_setprio(0);
      }
    }
    const int buf = c & 1;
    const bool more = c + 1 < nstages;
    if (more) stage_load(c + 1);
    const uint32_t *sBl = &sB[buf * Cfg::TILE + lane_row];
    const bool is_window = c == nfull;  // only possible for the last iteration
    const uint64_t Abase = Abase0 + (uint64_t)(uint32_t)stage_word0(c) * 8u;
    u32x8 a[TM];
    u32x8 b[TN];
    uint32_t aoff_cur = aoff_first;
    asm volatile("" : "+s"(aoff_cur));
#pragma unroll
    for (int i = 0; i < TM; ++i)
      asm volatile("s_load_dwordx8 %0, %1, %2" : "=s"(a[i]) : "s"(Abase), "s"(BNN_AOFF(i)));
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      b[j].lo = *reinterpret_cast<const u32x4 *>(&sBl[j * 64 * RS]);
      b[j].hi = *reinterpret_cast<const u32x4 *>(&sBl[j * 64 * RS + 4]);
    }
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+s"(a[0]), "+s"(a[1]), "+s"(a[2]), "+s"(a[3]), "+s"(a[4]), "+s"(a[5]), "+s"(a[6]), "+s"(a[7]));
    if (is_window) {
      // dwords already counted by the full chunks, and the bits past K, leave A as zeros
      int dw_done = 2 * (4 * nfull - (p.Kw64 - 4));
      asm volatile("" : "+s"(dw_done));  // the eight compares below stay here, not in registers across the loop
      const uint32_t m6 = (uint32_t)tail_mask, m7 = (uint32_t)(tail_mask >> 32);
#pragma unroll
      for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int d = 0; d < 8; ++d)
          if (d < dw_done) a[i][d] = 0u;
        a[i][6] &= m6;
        a[i][7] &= m7;
      }
    }
    uint32_t t0, t1;
#define BNN_BV(j, d) b[j][d]
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      if constexpr (YIELD) {
        if constexpr (TN == 8) BNN_GEMM_ROW_8(acc[i], a[i], BNN_BV, t0, t1);
        else if constexpr (TN == 4) BNN_GEMM_ROW_4(acc[i], a[i], BNN_BV, t0, t1);
        else if constexpr (TN == 2) BNN_GEMM_ROW_2(acc[i], a[i], BNN_BV, t0, t1);
        else BNN_GEMM_ROW_1(acc[i], a[i], BNN_BV, t0, t1);
      } else {
        if constexpr (TN == 8) BNN_GEMM_ROW_8_NY(acc[i], a[i], BNN_BV, t0, t1);
        else if constexpr (TN == 4) BNN_GEMM_ROW_4_NY(acc[i], a[i], BNN_BV, t0, t1);
        else if constexpr (TN == 2) BNN_GEMM_ROW_2_NY(acc[i], a[i], BNN_BV, t0, t1);
        else BNN_GEMM_ROW_1_NY(acc[i], a[i], BNN_BV, t0, t1);
      }
    }
#undef BNN_BV
    if (more) {
      stage_store(buf ^ 1, c + 1);  // that buffer was last read in chunk c-1, before the previous barrier
      __syncthreads();
    }
  }

  // ---- half chunk: the last two words of rows of 4*n + 2 words -------------------------------
  if (half) {
    const uint32_t *sBl = &sB[(nfull & 1) * Cfg::TILE + lane_row];
    const uint64_t Abase = Abase0 + (uint64_t)(uint32_t)(4 * nfull) * 8u;
    u32x4 a[TM];
    u32x4 b[TN];
    uint32_t aoff_cur = aoff_first;
    asm volatile("" : "+s"(aoff_cur));
#pragma unroll
    for (int i = 0; i < TM; ++i)
      asm volatile("s_load_dwordx4 %0, %1, %2" : "=s"(a[i]) : "s"(Abase), "s"(BNN_AOFF(i)));
#pragma unroll
    for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const u32x4 *>(&sBl[j * 64 * RS]);
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+s"(a[0]), "+s"(a[1]), "+s"(a[2]), "+s"(a[3]), "+s"(a[4]), "+s"(a[5]), "+s"(a[6]), "+s"(a[7]));
    const uint32_t m2 = (uint32_t)tail_mask, m3 = (uint32_t)(tail_mask >> 32);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      a[i][2] &= m2;
      a[i][3] &= m3;
    }
    uint32_t t0, t1;
#define BNN_BV(j, d) b[j][d]
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      if constexpr (YIELD) {
        if constexpr (TN == 8) BNN_GEMM_HALF_8(acc[i], a[i], BNN_BV, t0, t1);
        else if constexpr (TN == 4) BNN_GEMM_HALF_4(acc[i], a[i], BNN_BV, t0, t1);
        else if constexpr (TN == 2) BNN_GEMM_HALF_2(acc[i], a[i], BNN_BV, t0, t1);
        else BNN_GEMM_HALF_1(acc[i], a[i], BNN_BV, t0, t1);
      } else {
        if constexpr (TN == 8) BNN_GEMM_HALF_8_NY(acc[i], a[i], BNN_BV, t0, t1);
        else if constexpr (TN == 4) BNN_GEMM_HALF_4_NY(acc[i], a[i], BNN_BV, t0, t1);
        else if constexpr (TN == 2) BNN_GEMM_HALF_2_NY(acc[i], a[i], BNN_BV, t0, t1);
        else BNN_GEMM_HALF_1_NY(acc[i], a[i], BNN_BV, t0, t1);
      }
    }
#undef BNN_BV
  }

  // ---- rows of one or three words (K < 193): one dword at a time ----------------------------
  // B is already masked / zero-filled by the staging; A is masked here.
  if (slow_tail) {
    const uint32_t *sBl = &sB[(nfull & 1) * Cfg::TILE + lane_row];
    const int kd0 = nfull * KC;
    const int tb32 = p.Kbits & 31;
#pragma unroll 1
    for (int kd = kd0; kd < p.Kd; ++kd) {
      const uint32_t amask = (kd == p.Kd - 1 && tb32) ? ((1u << tb32) - 1u) : 0xffffffffu;
      uint32_t b[TN];
#pragma unroll
      for (int j = 0; j < TN; ++j) b[j] = sBl[j * 64 * RS + (kd - kd0)];
      uint32_t aoff_cur = aoff_first;
      asm volatile("" : "+s"(aoff_cur));
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const uint32_t a = Ac[(BNN_AOFF(i) >> 2) + kd] & amask;
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = popc_acc(a ^ b[j], acc[i][j]);
      }
    }
  }

  // ---- store ------------------------------------------------------------------------
  __builtin_amdgcn_s_setprio(3);
  if constexpr (EMODE == 0) {
    if constexpr (TN == 4 && WN == 1) {
      if (colperm) store_tile_x4(acc, m0, n0 + 4 * lane);
      else store_tile<TN>(acc, m0, n0 + lane);
    } else {
      store_tile<TN>(acc, m0, n0 + wn * 64 * TN + lane);
    }
  } else {
    // Binarizing epilogue.  Row m is output channel m; the workgroup's 8 * WM rows are one
    // 64-bit channel word (WM = 8), or one 32-bit half of it (WM = 4), of every pixel in its
    // tile.  Each lane turns its 8 channels into a byte per output pixel, the waves' bytes
    // meet in LDS, and one thread per pixel writes the assembled (half) word.
    const GemmParams BNN_CONST_AS *kp = (const GemmParams BNN_CONST_AS *)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(kp));
    const int M = kp->M, N = kp->N, Kformula = kp->Kformula;
    const float *const scale = kp->scale, *const bias = kp->bias;
    const int pool = kp->g.pool;
    uint64_t *const outp = kp->outp;
    const int cw_out = kp->cw_out;
    uint32_t bytes[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) bytes[j] = 0u;
    // The affine constants of the wave's 8 rows: wave-uniform, read through the constant address
    // space (scalar loads), all 16 requested before the first is used, rows past M re-reading row
    // M - 1.  (Loaded row by row inside the loop below they were 16 dependent vector loads, each
    // waited for: eight memory round trips at the end of every tile, during which the wave held
    // its slot without issuing.)
    typedef const float BNN_CONST_AS *cf32_ptr;
    const cf32_ptr cscale = (cf32_ptr)(uintptr_t)scale, cbias = (cf32_ptr)(uintptr_t)bias;
    float scr[TM], bir[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int mc = min(m0 + i, M - 1);
      scr[i] = cscale[mc];
      bir[i] = cbias[mc];
    }
    // Rows run from the last to the first so that each sign is shifted in with one add-with-carry
    // (byte = 2 * byte + bit).  K - 2*acc decreases in acc: the 2x2 max is K - 2*min(acc).
#pragma unroll
    for (int i = TM - 1; i >= 0; --i) {
      const int m = m0 + i;
      const bool row_ok = m < M;
      const float sc = row_ok ? scr[i] : 0.0f;
      const float bi = row_ok ? bir[i] : -1.0f;  // rows past M give bit 0
      if (pool) {
        int a = acc[i][0];
#pragma unroll
        for (int j = 1; j < TN; ++j) a = min(a, acc[i][j]);
        const float y = fmaf(sc, (float)(Kformula - 2 * a), bi);
        asm("v_cmp_le_f32 vcc, 0, %1\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc" : "+v"(bytes[0]) : "v"(y) : "vcc");
      } else {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const float y = fmaf(sc, (float)(Kformula - 2 * acc[i][j]), bi);
          asm("v_cmp_le_f32 vcc, 0, %1\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc" : "+v"(bytes[j]) : "v"(y) : "vcc");
        }
      }
    }
    __syncthreads();  // every wave is done reading the B tiles: LDS is reused for the output bytes
    uint8_t *sO = reinterpret_cast<uint8_t *>(sB);
    if (pool) {
      sO[lane * WM + wm] = (uint8_t)bytes[0];
    } else {
#pragma unroll
      for (int j = 0; j < TN; ++j) sO[(j * 64 + lane) * WM + wm] = (uint8_t)bytes[j];
    }
    __syncthreads();
    const int npix = pool ? 64 : 64 * TN;
    if (tid < npix) {
      // global pixel index: pooled window index, or column index (NHWC pixel order)
      const int64_t gp = pool ? (int64_t)ni * 64 + tid : (int64_t)n0 + tid;
      const int64_t limit = pool ? (int64_t)(N >> 2) : (int64_t)N;
      if (gp < limit) {
        if constexpr (WM == 8) {
          const uint2 w = *reinterpret_cast<const uint2 *>(&sO[tid * 8]);
          *reinterpret_cast<uint2 *>(outp + gp * cw_out + mi) = w;
        } else {
          // 32 channels: half of word (mi / 2); a last odd half past D is written as zeros
          const uint32_t w = *reinterpret_cast<const uint32_t *>(&sO[tid * 4]);
          uint32_t *o32 = reinterpret_cast<uint32_t *>(outp) + (gp * cw_out) * 2;
          o32[mi] = w;
          if (mi == kp->tilesM - 1 && (kp->tilesM & 1)) o32[mi + 1] = 0u;  // channels past D: pad bits 0
        }
      }
    }
  }
}


// ---- small problems: one independent wave per 8 x (64*TN) tile, no LDS, no barrier -------------
// When a problem has too few tiles to put two waves on every SIMD, the LDS-staged kernel is
// bound by its per-chunk latency chain (global load -> LDS -> barrier).  Here every lane reads
// its own columns' words straight from global memory into registers, DEPTH chunks ahead, and
// the wave never synchronises with anyone.  A is fetched with scalar loads as above.
// KS = 4: the four waves of a workgroup share ONE tile and split its K range (problems with
// fewer tiles than SIMDs but long rows); their partial counts are summed through LDS.
template <int TN, int DEPTH, int YIELD, int KS>
__global__ __launch_bounds__(256) void xnor_gemm_direct_kernel(GemmParams p) {
  static_assert(KS == 1 || KS == 4, "one tile per wave, or one per workgroup");
  __shared__ int sRed[KS == 4 ? 3 * TM * TN * 64 : 1];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const uint32_t wid = KS == 4 ? blockIdx.x : blockIdx.x * 4u + (uint32_t)wave;  // tile index, M fastest
  const int mi = (int)(wid % (uint32_t)p.tilesM);
  const int ni = (int)(wid / (uint32_t)p.tilesM);
  if (ni >= p.tilesN) return;
  const int m0 = mi * TM;
  const int nbase = ni * 64 * TN + lane;

  uint32_t aoffb[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    int m = m0 + i;
    m = m < p.M ? m : p.M - 1;
    aoffb[i] = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)m * (uint32_t)p.lda32 * 4u));
  }
  const uint32_t Abase_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)p.A);
  const uint32_t Abase_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uintptr_t)p.A >> 32));
  const uint64_t Abase0 = ((uint64_t)Abase_hi << 32) | (uint64_t)Abase_lo;
  const cu32_ptr Ac = (cu32_ptr)(uintptr_t)p.A;

  // this lane's TN rows of B (clamped: columns past N recompute column N-1 and are not stored)
  const uint64_t *brow[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    int n = nbase + j * 64;
    n = n < p.N ? n : p.N - 1;
    brow[j] = p.B + (int64_t)n * p.ldb;
  }

  int acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = 0;

  const int nfull_all = p.Kbits / (32 * KC);
  // this wave's range of full chunks: [cb, cb + nfull)
  const int per = KS == 4 ? (nfull_all + 3) / 4 : nfull_all;
  const int cb = KS == 4 ? min(wave * per, nfull_all) : 0;
  const int nfull = KS == 4 ? min(per, nfull_all - cb) : nfull_all;
  auto load_b = [&](u32x8 (&b)[TN], int cl) {
    const int c = cb + cl;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const uint64_t *src = brow[j] + 4 * c;
      if (p.b_vec16) {
        b[j].lo = *reinterpret_cast<const u32x4 *>(src);
        b[j].hi = *reinterpret_cast<const u32x4 *>(src + 2);
      } else {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const uint2 v = *reinterpret_cast<const uint2 *>(src + w);
          b[j][2 * w] = v.x;
          b[j][2 * w + 1] = v.y;
        }
      }
    }
  };
  auto compute = [&](u32x8 (&b)[TN], int cl) {
    const uint64_t Abase = Abase0 + (uint64_t)(uint32_t)(cb + cl) * 32u;
    u32x8 a[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i)
      asm volatile("s_load_dwordx8 %0, %1, %2" : "=s"(a[i]) : "s"(Abase), "s"(aoffb[i]));
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+s"(a[0]), "+s"(a[1]), "+s"(a[2]), "+s"(a[3]), "+s"(a[4]), "+s"(a[5]), "+s"(a[6]), "+s"(a[7]));
    uint32_t t0, t1;
#define BNN_BV(j, d) b[j][d]
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      if constexpr (YIELD) {
        if constexpr (TN == 2) BNN_GEMM_ROW_2(acc[i], a[i], BNN_BV, t0, t1);
        else BNN_GEMM_ROW_1(acc[i], a[i], BNN_BV, t0, t1);
      } else {
        if constexpr (TN == 2) BNN_GEMM_ROW_2_NY(acc[i], a[i], BNN_BV, t0, t1);
        else BNN_GEMM_ROW_1_NY(acc[i], a[i], BNN_BV, t0, t1);
      }
    }
#undef BNN_BV
  };

  // software pipeline over full chunks, DEPTH loads in flight (slots indexed statically)
  u32x8 bq[DEPTH][TN];
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

  // bits past the last full chunk: one dword at a time, both operands masked (first wave only
  // when the K range is split)
  if (KS == 1 || wave == 0) {
    const int kd0 = nfull_all * KC;
    const int tb32 = p.Kbits & 31;
    const uint32_t *b32[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) b32[j] = reinterpret_cast<const uint32_t *>(brow[j]);
#pragma unroll 1
    for (int kd = kd0; kd < p.Kd; ++kd) {
      const uint32_t mask = (kd == p.Kd - 1 && tb32) ? ((1u << tb32) - 1u) : 0xffffffffu;
      uint32_t b[TN];
#pragma unroll
      for (int j = 0; j < TN; ++j) b[j] = b32[j][kd] & mask;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const uint32_t a = Ac[(aoffb[i] >> 2) + kd] & mask;
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = popc_acc(a ^ b[j], acc[i][j]);
      }
    }
  }
  if constexpr (KS == 4) {
    // every wave of the workgroup is here (the early return above is per workgroup)
    if (wave > 0) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) sRed[((wave - 1) * TM * TN + i * TN + j) * 64 + lane] = acc[i][j];
    }
    __syncthreads();
    if (wave > 0) return;
#pragma unroll
    for (int w = 0; w < 3; ++w)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] += sRed[(w * TM * TN + i * TN + j) * 64 + lane];
  }
  store_tile<TN>(acc, m0, nbase);
}

// ---- few outputs, long rows: K split over the waves of a workgroup -----------------------------
// A fully-connected layer (a few hundred rows of activations against thousands of filter rows)
// has too few 8 x 64 tiles to give every SIMD its waves, and when every wave reads its own copy
// of B straight from memory, as above, B crosses the L2 once per 8 rows of A: at M = 256 that is
// 32 times the matrix, and that traffic, not the arithmetic, bounds the kernel.  Here a wave
// keeps its chunk of B in registers while it walks 8 * TMG rows of A (8 at a time through the
// scalar loads), so B is read once per 8 * TMG rows, and the parallelism lost to the taller tile
// comes back from the reduction axis: the KS waves of a workgroup share one tile, each takes a
// contiguous range of K chunks, and their partial counts (additive: section 3.2's sum over the
// reduction axis) meet in LDS, where every wave adds up and stores its share of the rows.
template <int TMG, int KS, int YIELD>
__global__ __launch_bounds__(64 * KS) void xnor_gemm_splitk_kernel(GemmParams p) {
  constexpr int DEPTH = 2;
  __shared__ int sRed[KS * TMG * TM * 64];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const uint32_t tile = blockIdx.x;  // M fastest: consecutive workgroups share a B tile
  const int mi = (int)(tile % (uint32_t)p.tilesM);
  const int ni = (int)(tile / (uint32_t)p.tilesM);
  const int m0 = mi * TM * TMG;
  const int nbase = ni * 64 + lane;

  const uint32_t arow_bytes = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)p.lda32 * 4u));
  const uint32_t aoff_max = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)(p.M - 1) * (uint32_t)p.lda32 * 4u));
  const uint32_t aoff_tile = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)min(m0, p.M - 1) * (uint32_t)p.lda32 * 4u));
  const uint32_t Abase_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)p.A);
  const uint32_t Abase_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uintptr_t)p.A >> 32));
  const uint64_t Abase0 = ((uint64_t)Abase_hi << 32) | (uint64_t)Abase_lo;
  const cu32_ptr Ac = (cu32_ptr)(uintptr_t)p.A;

  // this lane's row of B (clamped: columns past N recompute column N-1 and are not stored)
  const uint64_t *brow = p.B + (int64_t)min(nbase, p.N - 1) * p.ldb;

  int acc[TMG][TM][1];
#pragma unroll
  for (int g = 0; g < TMG; ++g)
#pragma unroll
    for (int i = 0; i < TM; ++i) acc[g][i][0] = 0;

  const int nfull_all = p.Kbits / (32 * KC);
  const int per = (nfull_all + KS - 1) / KS;
  const int cb = min(wave * per, nfull_all);     // this wave's chunks: [cb, cb + nfull)
  const int nfull = min(per, nfull_all - cb);
  auto load_b = [&](u32x8 &b, int cl) {
    const uint64_t *src = brow + 4 * (cb + cl);
    if (p.b_vec16) {
      b.lo = *reinterpret_cast<const u32x4 *>(src);
      b.hi = *reinterpret_cast<const u32x4 *>(src + 2);
    } else {
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint2 v = *reinterpret_cast<const uint2 *>(src + w);
        b[2 * w] = v.x;
        b[2 * w + 1] = v.y;
      }
    }
  };
  auto compute = [&](const u32x8 &bv, int cl) {
    const uint64_t Abase = Abase0 + (uint64_t)(uint32_t)(cb + cl) * 32u;
#pragma unroll
    for (int g = 0; g < TMG; ++g) {
      u32x8 a[TM];
      uint32_t aoff_cur = aoff_tile + (uint32_t)(g * TM) * arow_bytes;
      asm volatile("" : "+s"(aoff_cur));
#pragma unroll
      for (int i = 0; i < TM; ++i)
        asm volatile("s_load_dwordx8 %0, %1, %2" : "=s"(a[i]) : "s"(Abase), "s"(BNN_AOFF(i)));
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+s"(a[0]), "+s"(a[1]), "+s"(a[2]), "+s"(a[3]), "+s"(a[4]), "+s"(a[5]), "+s"(a[6]), "+s"(a[7]));
      uint32_t t0, t1;
#define BNN_BV(j, d) bv[d]
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        if constexpr (YIELD) BNN_GEMM_ROW_1(acc[g][i], a[i], BNN_BV, t0, t1);
        else BNN_GEMM_ROW_1_NY(acc[g][i], a[i], BNN_BV, t0, t1);
      }
#undef BNN_BV
    }
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

  // bits past the last full chunk: one dword at a time, both operands masked (first wave only)
  if (wave == 0) {
    const int kd0 = nfull_all * KC;
    const int tb32 = p.Kbits & 31;
    const uint32_t *b32 = reinterpret_cast<const uint32_t *>(brow);
#pragma unroll 1
    for (int kd = kd0; kd < p.Kd; ++kd) {
      const uint32_t mask = (kd == p.Kd - 1 && tb32) ? ((1u << tb32) - 1u) : 0xffffffffu;
      const uint32_t b = b32[kd] & mask;
#pragma unroll
      for (int g = 0; g < TMG; ++g) {
        uint32_t aoff_cur = aoff_tile + (uint32_t)(g * TM) * arow_bytes;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          const uint32_t a = Ac[(BNN_AOFF(i) >> 2) + kd] & mask;
          acc[g][i][0] = popc_acc(a ^ b, acc[g][i][0]);
        }
      }
    }
  }

  // partial counts -> LDS [slice][row][lane]; every wave then sums the row groups g = wave, wave + KS, ...
#pragma unroll
  for (int g = 0; g < TMG; ++g)
#pragma unroll
    for (int i = 0; i < TM; ++i) sRed[((wave * TMG + g) * TM + i) * 64 + lane] = acc[g][i][0];
  __syncthreads();
#pragma unroll
  for (int g0 = 0; g0 < TMG; g0 += KS) {
    const int g = g0 + wave;
    if (g < TMG && m0 + g * TM < p.M) {  // wave-uniform
      int tot[TM][1];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        int t = 0;
#pragma unroll
        for (int k = 0; k < KS; ++k) t += sRed[((k * TMG + g) * TM + i) * 64 + lane];
        tot[i][0] = t;
      }
      store_tile<1>(tot, m0 + g * TM, nbase);
    }
  }
}

// ---- host side ----------------------------------------------------------------------
template <int TN, int WM, int WN, int MINW, int BMODE, int EMODE, int YIELD>
static bnn_status launch_one(GemmParams &p, hipStream_t s, int kid) {
  using Cfg = GemmCfg<TN, WM, WN>;
  // the last resident set: MINW waves per SIMD, 4 SIMDs per compute unit
  const int64_t resident = (int64_t)(MINW * 4 / (Cfg::THREADS / 64)) * p.n_cu;
  const int64_t nb = (int64_t)p.tilesM * p.tilesN;
  p.prio_from = (int)(nb > resident ? nb - resident : 0);
  ProfScope ps(kid, s);
  hipLaunchKernelGGL((xnor_gemm_kernel<TN, WM, WN, MINW, BMODE, EMODE, YIELD>),
                     dim3((unsigned)(p.tilesM * p.tilesN)), dim3(Cfg::THREADS), 0, s, p);
  return launch_status();
}

template <int TN, int WM, int WN, int MINW>
static bnn_status launch_cfg(GemmParams &p, int bmode, int emode, hipStream_t s, int kid) {
  using Cfg = GemmCfg<TN, WM, WN>;
  p.tilesM = (p.M + Cfg::BM - 1) / Cfg::BM;
  p.tilesN = (p.N + Cfg::BN - 1) / Cfg::BN;
  const int64_t blocks = (int64_t)p.tilesM * p.tilesN;
  if (blocks > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  // The one-cycle yields after each xor/popcount pair pay off only when at least two waves
  // share a SIMD (4 per compute unit); with fewer they cost issue slots.
  const int64_t waves = blocks * (Cfg::THREADS / 64);
  const bool yield = waves >= 2 * 4 * (int64_t)p.n_cu;
  // 256-column tiles writing int32 / fp32: four consecutive columns per lane and 16-byte stores where
  // every group of four columns is whole, inside one image and 16-byte aligned
  p.colperm = (emode == 0 && TN == 4 && WN == 1 && (p.N & 3) == 0 && (!p.C || (p.ldc & 3) == 0) &&
               (!p.Y || (p.ldy & 3) == 0) && (p.img_stride == 0 || ((p.OHW & 3u) == 0 && (p.img_stride & 3) == 0)))
                  ? 1
                  : 0;
  if constexpr ((TN == 4 || TN == 2) && (WM == 8 || WM == 4) && WN == 1) {
    if (emode == 1) {
      if (bmode == 0 || (p.g.pool && TN != 4)) return BNN_ERR_UNSUPPORTED;
      if (bmode == 2)
        return yield ? launch_one<TN, WM, WN, MINW, 2, 1, 1>(p, s, kid) : launch_one<TN, WM, WN, MINW, 2, 1, 0>(p, s, kid);
      return yield ? launch_one<TN, WM, WN, MINW, 1, 1, 1>(p, s, kid) : launch_one<TN, WM, WN, MINW, 1, 1, 0>(p, s, kid);
    }
  }
  if (emode != 0) return BNN_ERR_UNSUPPORTED;
  if (bmode == 2)
    return yield ? launch_one<TN, WM, WN, MINW, 2, 0, 1>(p, s, kid) : launch_one<TN, WM, WN, MINW, 2, 0, 0>(p, s, kid);
  if (bmode == 1)
    return yield ? launch_one<TN, WM, WN, MINW, 1, 0, 1>(p, s, kid) : launch_one<TN, WM, WN, MINW, 1, 0, 0>(p, s, kid);
  return yield ? launch_one<TN, WM, WN, MINW, 0, 0, 1>(p, s, kid) : launch_one<TN, WM, WN, MINW, 0, 0, 0>(p, s, kid);
}

template <int TN>
static bnn_status launch_direct(GemmParams &p, hipStream_t s, int ksplit = -1) {  // ksplit: -1 heuristic, 0 off, 1 on
  p.tilesM = (p.M + TM - 1) / TM;
  p.tilesN = (p.N + 64 * TN - 1) / (64 * TN);
  const int64_t waves = (int64_t)p.tilesM * p.tilesN;
  if (waves > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  ProfScope ps(KID_XNOR_GEMM_SMALL, s);
  const int64_t simds = 4 * (int64_t)p.n_cu;
  if constexpr (TN == 1) {
    // fewer tiles than SIMDs and at least four chunks per wave after the split: four waves per tile
    if (ksplit > 0 || (ksplit < 0 && waves < simds && p.Kbits / (32 * KC) >= 16)) {
      if (4 * waves >= 2 * simds)
        hipLaunchKernelGGL((xnor_gemm_direct_kernel<1, 4, 1, 4>), dim3((unsigned)waves), dim3(256), 0, s, p);
      else
        hipLaunchKernelGGL((xnor_gemm_direct_kernel<1, 4, 0, 4>), dim3((unsigned)waves), dim3(256), 0, s, p);
      return launch_status();
    }
  }
  const int64_t blocks = (waves + 3) / 4;
  if (waves >= 2 * simds)
    hipLaunchKernelGGL((xnor_gemm_direct_kernel<TN, 4, 1, 1>), dim3((unsigned)blocks), dim3(256), 0, s, p);
  else
    hipLaunchKernelGGL((xnor_gemm_direct_kernel<TN, 4, 0, 1>), dim3((unsigned)blocks), dim3(256), 0, s, p);
  return launch_status();
}

int device_cu_count() {
  // one slot per device id; concurrent first calls write the same value
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cached[dev] = n;
  }
  return cached[dev];
}

template <int TMG, int KS>
static bnn_status launch_splitk(GemmParams &p, hipStream_t s) {
  p.tilesM = (p.M + TM * TMG - 1) / (TM * TMG);
  p.tilesN = (p.N + 63) / 64;
  const int64_t tiles = (int64_t)p.tilesM * p.tilesN;
  if (tiles > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  ProfScope ps(KID_XNOR_GEMM_SMALL, s);
  if (tiles * KS >= 2 * 4 * (int64_t)p.n_cu)
    hipLaunchKernelGGL((xnor_gemm_splitk_kernel<TMG, KS, 1>), dim3((unsigned)tiles), dim3(64 * KS), 0, s, p);
  else
    hipLaunchKernelGGL((xnor_gemm_splitk_kernel<TMG, KS, 0>), dim3((unsigned)tiles), dim3(64 * KS), 0, s, p);
  return launch_status();
}

static bnn_status launch_splitk_by(GemmParams &p, int tmg, int ks, hipStream_t s) {
  if (tmg == 4) {
    if (ks == 8) return launch_splitk<4, 8>(p, s);
    if (ks == 4) return launch_splitk<4, 4>(p, s);
    if (ks == 2) return launch_splitk<4, 2>(p, s);
  } else if (tmg == 2) {
    if (ks == 8) return launch_splitk<2, 8>(p, s);
    if (ks == 4) return launch_splitk<2, 4>(p, s);
    if (ks == 2) return launch_splitk<2, 2>(p, s);
  }
  return BNN_ERR_UNSUPPORTED;
}

bnn_status run_gemm(GemmParams &p, int bmode, int emode, hipStream_t s, const GemmTune &tune) {
  int cfg = tune.cfg;
  p.n_cu = device_cu_count();
  {
    const bool planes = p.img_stride != 0;
    const bool c_ok = !p.C || (((uintptr_t)p.C & 127u) == 0 && (planes ? (p.OHW % 32u) == 0 : (p.ldc % 32) == 0));
    const bool y_ok = !p.Y || (((uintptr_t)p.Y & 127u) == 0 && (planes ? (p.OHW % 32u) == 0 : (p.ldy % 32) == 0));
    p.nt_store = (c_ok && y_ok) ? 1 : 0;
  }
  const int64_t full = 2 * (int64_t)p.n_cu;  // tiles that give every compute unit two workgroups
  if (bmode == 1 && emode == 0 && p.g.pool == 0 && p.g.kH == 1 && p.g.kW == 1 && p.g.sH == 1 && p.g.sW == 1 &&
      p.g.pH == 0 && p.g.pW == 0) {
    // a stride-1 pointwise convolution over a packed image has nothing to gather: its patch
    // matrix is the packed image itself
    bmode = 0;
    p.B = p.g.act;
    p.ldb = p.g.Cw;
    p.b_vec16 = (p.g.Cw & 1) == 0 ? 1 : 0;
  }
  if (bmode == 0 && emode == 0 && (cfg < 0 || (cfg >= 10 && cfg <= 12)) && lowk_applicable(p) &&
      ((int64_t)p.M + 31) / 32 <= 65535) {
    // rows of two or four words: bound by the store, see gemm_lowk.hip.  As many rows per wave
    // (32, 16 or 8) as still leave every compute unit a workgroup.
    const int64_t ctiles = ((int64_t)p.N + 255) / 256;
    const int groups = cfg == 12 ? 4 : cfg == 11 ? 2 : cfg == 10 ? 1
                       : (ctiles * (((int64_t)p.M + 127) / 128) >= (int64_t)p.n_cu  ? 4
                          : ctiles * (((int64_t)p.M + 63) / 64) >= (int64_t)p.n_cu ? 2
                                                                                    : 1);
    return launch_lowk(p, groups, s);
  }
  if (cfg >= 10 && cfg <= 12) cfg = -1;
  if (bmode == 1 && (cfg == 19 || cfg == 20) && latency_applicable(p)) return launch_latency(p, emode, cfg == 19 ? 4 : 2, s);
  if (cfg == 19 || cfg == 20) cfg = -1;
  if (bmode == 1 && cfg < 0 && latency_applicable(p)) {
    // Few output pixels (small batches, late layers): the latency form, see gemm_latency.hip.  Its
    // workgroups fill a compute unit each, so it wins while there is at most one per compute unit
    // (measured on the layers of the stack at batch 1 to 64: 1.5 to 2.2 times faster there, slower
    // beyond); pooled layers, whose throughput tile is four columns wide, up to two per unit.
    const int64_t lt = (((int64_t)p.M + 31) / 32) * (((int64_t)p.N + 63) / 64);
    if (lt <= (int64_t)p.n_cu) return launch_latency(p, emode, 4, s);
    if (p.g.pool && lt <= 2 * (int64_t)p.n_cu) return launch_latency(p, emode, 2, s);
  }
  if (bmode == 1 && tune.lean) {
    // lean gather: 16-byte pieces never straddle a tap (even Cw), one validity bit per tap in a
    // 32-bit mask, 32-bit byte offsets into the packed image
    const int64_t taps = (int64_t)p.g.kH * p.g.kW;
    const int64_t img_bytes = (int64_t)p.g.Nimg * p.g.H * p.g.W * p.g.Cw * 8;
    if ((p.g.Cw & 1) == 0 && taps <= 32 && img_bytes <= 0xffffffffLL && (p.Kw64 + 3) / 4 <= LEAN_MAX_STAGES) bmode = 2;
  }
  if (bmode == 0 && emode == 0 && (cfg == 7 || cfg == 8 || cfg < 0)) {
    // Too few 32 x 128 tiles to give every SIMD two waves of the LDS-staged kernel: use
    // independent waves on 8 x 128 (or 8 x 64) tiles instead.
    const int64_t t32 = (int64_t)((p.M + 31) / 32) * ((p.N + 127) / 128);
    const int64_t w128 = (int64_t)((p.M + 7) / 8) * ((p.N + 127) / 128);
    const int nchunks = p.Kbits / (32 * KC);
    if (cfg < 0 && t32 < full && nchunks >= 16 && ((int64_t)p.M + 32) * p.lda32 * 4 <= 0xffffffffLL) {
      // long rows, few outputs: the tallest tile (32, 16 or 8 rows per wave, K split 8 / 8 / 4 ways over
      // the waves of a workgroup) that still gives every SIMD two waves; if none does, the one
      // with the most waves, the lower tile on a tie.  Measured: 256 x 4096 x 4096 12.8 -> 10.9 us,
      // 256 x 1024 x 8192 8.4 -> 7.9 us per launch inside a replayed graph (an empty launch: 3.3 us).
      const int64_t ct = ((int64_t)p.N + 63) / 64;
      const int64_t w4 = (((int64_t)p.M + 31) / 32) * ct * 8, w2 = (((int64_t)p.M + 15) / 16) * ct * 8,
                    w1 = (((int64_t)p.M + 7) / 8) * ct * 4;
      const int64_t want = 2 * 4 * (int64_t)p.n_cu;
      if (w4 >= want) return launch_splitk<4, 8>(p, s);
      if (w2 >= want) return launch_splitk<2, 8>(p, s);
      if (w1 < want && w2 > w1 && w2 >= w4) return launch_splitk<2, 8>(p, s);
      if (w1 < want && w4 > w1 && w4 > w2) return launch_splitk<4, 8>(p, s);
      return launch_direct<1>(p, s, 1);
    }
    if (cfg == 8 || (cfg < 0 && t32 < full && w128 >= 4 * full)) return launch_direct<2>(p, s);
    if (cfg == 7 || (cfg < 0 && t32 < full)) return launch_direct<1>(p, s, cfg == 7 ? 0 : -1);
  }
  if (bmode == 0 && emode == 0 && cfg == 9) return launch_direct<1>(p, s, 1);  // forced K split
  if (bmode == 0 && emode == 0 && cfg >= 13 && cfg <= 18) {
    static const int tm[6] = {4, 4, 2, 2, 4, 2}, ks[6] = {4, 8, 8, 4, 2, 2};
    return launch_splitk_by(p, tm[cfg - 13], ks[cfg - 13], s);
  }
  // a forced value this call cannot use (the one-wave kernels read an explicit B and store
  // int32 / fp32; anything that is not a tile configuration) selects the heuristic
  if (cfg == 7 || cfg == 8 || cfg == 9 || cfg == 5 || cfg == 0 || cfg > 9) cfg = -1;
  if (emode == 1) {
    // tiles the packed epilogue is written for: 64 x 256 (3), 64 x 128 (6), 32 x 256 (1), 32 x 128 (4);
    // pooling needs four columns per lane (3 or 1)
    const bool ok = p.g.pool ? (cfg == 3 || cfg == 1) : (cfg == 3 || cfg == 6 || cfg == 1 || cfg == 4);
    // 64 x 256 is the fastest tile when a compute unit gets more than two of them; with two or
    // fewer, 32 x 256 (four waves per workgroup, twice as many workgroups) is as fast or faster
    const int64_t t256 = (int64_t)((p.M + 63) / 64) * ((p.N + 255) / 256);
    // ... and without pooling 32 x 128 (again twice as many workgroups) while 32 x 256 would leave
    // a compute unit two workgroups or fewer
    const int64_t t32x256 = (int64_t)((p.M + 31) / 32) * ((p.N + 255) / 256);
    if (!ok) cfg = (!p.g.pool && t32x256 <= full) ? 4 : (t256 <= full ? 1 : 3);
  }
  if (cfg < 0) {
    // Measured on MI355X: 64 x 256 (TN = 4, eight waves per workgroup, six per SIMD) is the
    // fastest tile when there are enough of them; smaller problems take finer tiles so that
    // every CU has work.
    const int64_t t256 = (int64_t)((p.M + 63) / 64) * ((p.N + 255) / 256);
    const int64_t t128 = (int64_t)((p.M + 63) / 64) * ((p.N + 127) / 128);
    const int64_t t32 = (int64_t)((p.M + 31) / 32) * ((p.N + 127) / 128);
    cfg = (p.M >= 64 && t256 >= full) ? 3 : (p.M >= 64 && t128 >= full) ? 6 : (t32 >= full ? 4 : 2);
  }
  switch (cfg) {
    case 1: return launch_cfg<4, 4, 1, 4>(p, bmode, emode, s, KID_XNOR_GEMM);        // 32 x 256
    case 2: return launch_cfg<1, 4, 1, 4>(p, bmode, emode, s, KID_XNOR_GEMM_SMALL);  // 32 x 64
    case 3: return launch_cfg<4, 8, 1, 6>(p, bmode, emode, s, KID_XNOR_GEMM);        // 64 x 256
    case 4: return launch_cfg<2, 4, 1, 4>(p, bmode, emode, s, KID_XNOR_GEMM);        // 32 x 128
    case 6: return launch_cfg<2, 8, 1, 4>(p, bmode, emode, s, KID_XNOR_GEMM);        // 64 x 128
    default: return BNN_ERR_UNSUPPORTED;
  }
}

static bnn_status gemm_common(const uint64_t *A, int64_t lda, const uint64_t *B, int64_t ldb, int64_t M, int64_t N,
                              int64_t K, int32_t *C, int64_t ldc, float *Y, int64_t ldy, const float *scale,
                              const float *bias, bnn_ch_axis axis, void *stream, const GemmTune &tune = GemmTune()) {
  if (M < 0 || N < 0 || K <= 0) return BNN_ERR_SHAPE;
  const int64_t Kw = bnn_packed_words(K);
  if (lda < Kw || ldb < Kw) return BNN_ERR_STRIDE;
  if (C && ldc < N) return BNN_ERR_STRIDE;
  if (Y && ldy < N) return BNN_ERR_STRIDE;
  if (M == 0 || N == 0) return BNN_OK;
  if (!A || !B || (!C && !Y)) return BNN_ERR_NULL;
  if (Y && (!scale || !bias)) return BNN_ERR_NULL;
  if (Y && axis != BNN_CH_ROW && axis != BNN_CH_COL) return BNN_ERR_SHAPE;
  if (!aligned16(A) || !aligned16(B) || (C && !aligned16(C)) || (Y && !aligned16(Y))) return BNN_ERR_ALIGN;
  // column indices are ints computed on N rounded up to the tile width (at most 256)
  if (M > 0x7fffffffLL || N > 0x7fffffffLL - 256 || K > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  if (M * 8 * lda > 0xffffffffLL) return BNN_ERR_UNSUPPORTED;  // 32-bit byte offsets into A
  GemmParams p = {};
  p.A = reinterpret_cast<const uint32_t *>(A);
  p.B = B;
  p.lda32 = 2 * lda;
  p.ldb = ldb;
  p.M = (int)M;
  p.N = (int)N;
  p.Kbits = (int)K;
  p.Kformula = (int)K;
  p.Kd = (int)((K + 31) / 32);
  p.Kw64 = (int)Kw;
  p.b_vec16 = (ldb % 2 == 0) ? 1 : 0;
  p.C = C;
  p.Y = Y;
  p.ldc = ldc;
  p.ldy = ldy;
  p.scale = scale;
  p.bias = bias;
  p.axis = (int)axis;
  p.OHW = 0x7fffffffu;
  p.divOHW = FastDiv(0x7fffffffu);
  p.img_stride = 0;
  return run_gemm(p, 0, 0, (hipStream_t)stream, tune);
}

}  // namespace bnn

using namespace bnn;

extern "C" bnn_status bnn_xnor_gemm(const uint64_t *A, int64_t lda, const uint64_t *B, int64_t ldb, int32_t *C,
                                    int64_t ldc, int64_t M, int64_t N, int64_t K, void *stream) {
  if (M > 0 && N > 0 && K > 0 && !C) return BNN_ERR_NULL;
  return gemm_common(A, lda, B, ldb, M, N, K, C, ldc, nullptr, 0, nullptr, nullptr, BNN_CH_NONE, stream);
}

extern "C" bnn_status bnn_xnor_gemm_epilogue(const uint64_t *A, int64_t lda, const uint64_t *B, int64_t ldb, int64_t M,
                                             int64_t N, int64_t K, int32_t *C, int64_t ldc, float *Y, int64_t ldy,
                                             const float *scale, const float *bias, bnn_ch_axis axis, void *stream) {
  return gemm_common(A, lda, B, ldb, M, N, K, C, ldc, Y, ldy, scale, bias, axis, stream);
}

// Declared in bnn_testing.h: the same call with the tile configuration chosen by the caller.
extern "C" bnn_status bnn_testing_xnor_gemm_epilogue(const uint64_t *A, int64_t lda, const uint64_t *B, int64_t ldb,
                                                     int64_t M, int64_t N, int64_t K, int32_t *C, int64_t ldc,
                                                     float *Y, int64_t ldy, const float *scale, const float *bias,
                                                     bnn_ch_axis axis, int cfg, void *stream) {
  GemmTune tune;
  tune.cfg = cfg;
  return gemm_common(A, lda, B, ldb, M, N, K, C, ldc, Y, ldy, scale, bias, axis, stream, tune);
}
