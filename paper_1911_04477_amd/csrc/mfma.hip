// ABLATION, not the main path: the same binarized GEMM on the matrix cores.
//
// CDNA4 has no 1-bit MFMA, so each packed bit is expanded to an int8 (0 or 1) on the fly and
// V_MFMA_I32_32X32X32_I8 computes S[m,n] = sum_k a_k * b_k, the number of positions where
// both operands are +1.  With pa, pb the +1 counts of the two rows,
//     popcount(a XOR b) = pa + pb - 2*S   and   C = K - 2*popcount = K - 2*pa - 2*pb + 4*S,
// which is bit-identical to the XOR-popcount result.  The operands cost 8x the bytes of the
// packed form inside the CU (LDS), and the expansion itself runs on the VALU.
//
// Workgroup: 256 threads = 4 waves, tile 128 x 128, K consumed 64 bits at a time.  Thread t
// owns one row of the tile (A rows for t < 128, B rows after), loads that row's next 64-bit
// word, counts its ones, expands it to 64 bytes and stores them to LDS (row stride 80 bytes:
// conflict-free 16-byte accesses).  Each wave multiplies a 64 x 64 sub-tile: 2 x 2 blocks of
// 32 x 32, two K-steps of 32 per chunk.
#include "common.h"
#include "bnn_testing.h"

namespace bnn {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int MF_BM = 128, MF_BN = 128, MF_RS = 80;  // bytes per LDS row (64 + 16 pad)

struct MfmaParams {
  const uint64_t *A, *B;
  int64_t lda, ldb, ldc;
  int32_t *C;
  int M, N, K, Kw;
  int tilesM;
};

__device__ __forceinline__ void expand_store(uint64_t word, uint8_t *dst) {
  // nibble -> four bytes of 0/1: bit j of the nibble lands in byte j
  const uint32_t lo = (uint32_t)word, hi = (uint32_t)(word >> 32);
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    v4i v;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int nib_idx = g * 4 + e;  // nibble index 0..15
      const uint32_t src = nib_idx < 8 ? lo : hi;
      const uint32_t nib = (src >> ((nib_idx & 7) * 4)) & 0xFu;
      v[e] = (int)(__umul24(nib, 0x204081u) & 0x01010101u);
    }
    *reinterpret_cast<v4i *>(dst + g * 16) = v;
  }
}

__global__ __launch_bounds__(256, 2) void xnor_gemm_mfma_i8_kernel(MfmaParams p) {
  __shared__ __attribute__((aligned(16))) uint8_t sT[2][(MF_BM + MF_BN) * MF_RS];
  __shared__ int sPop[MF_BM + MF_BN];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int mi = blockIdx.x % p.tilesM, ni = blockIdx.x / p.tilesM;
  const int m0 = mi * MF_BM, n0 = ni * MF_BN;

  // this thread's row of the tile
  const bool isA = tid < MF_BM;
  const int grow = isA ? m0 + tid : n0 + (tid - MF_BM);
  const bool row_ok = isA ? grow < p.M : grow < p.N;
  const uint64_t *rowp = isA ? p.A + (int64_t)grow * p.lda : p.B + (int64_t)grow * p.ldb;
  const int tail = p.K & 63;
  const uint64_t tail_mask = tail ? ((1ull << tail) - 1ull) : ~0ull;
  auto load_word = [&](int c) -> uint64_t {
    uint64_t w = 0;
    if (row_ok && c < p.Kw) {
      w = rowp[c];
      if (c == p.Kw - 1) w &= tail_mask;
    }
    return w;
  };

  v16i acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0;

  int pop = 0;
  uint64_t cur = load_word(0);
  pop += __popcll(cur);
  expand_store(cur, &sT[0][tid * MF_RS]);
  __syncthreads();

  const int arow = (64 * wm + (lane & 31)) * MF_RS + 16 * (lane >> 5);
  const int brow = (MF_BM + 64 * wn + (lane & 31)) * MF_RS + 16 * (lane >> 5);

  for (int c = 0; c < p.Kw; ++c) {
    const int buf = c & 1;
    const bool more = c + 1 < p.Kw;
    uint64_t nxt = 0;
    if (more) nxt = load_word(c + 1);
    const uint8_t *T = sT[buf];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      v4i a[2], b[2];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) a[mb] = *reinterpret_cast<const v4i *>(T + arow + mb * 32 * MF_RS + ks * 32);
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) b[nb] = *reinterpret_cast<const v4i *>(T + brow + nb * 32 * MF_RS + ks * 32);
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
          acc[mb][nb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[mb], b[nb], acc[mb][nb], 0, 0, 0);
    }
    if (more) {
      pop += __popcll(nxt);
      expand_store(nxt, &sT[buf ^ 1][tid * MF_RS]);  // last read two iterations ago, before the previous barrier
      __syncthreads();
    }
  }

  sPop[tid] = pop;
  __syncthreads();

  // D[i][j] of a 32x32 block: lane l holds column j = l % 32; register r holds row
  // i = 8*(r/4) + 4*(l/32) + (r%4).
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const int nl = 64 * wn + 32 * nb + (lane & 31);
      const int n = n0 + nl;
      if (n >= p.N) continue;
      const int pb = sPop[MF_BM + nl];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int ml = 64 * wm + 32 * mb + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        const int m = m0 + ml;
        if (m < p.M) p.C[(int64_t)m * p.ldc + n] = p.K - 2 * (sPop[ml] + pb) + 4 * acc[mb][nb][r];
      }
    }
}

// ---- the same ablation on the 4-bit floating-point matrix instruction ------------------------
// V_MFMA_SCALE_F32_32X32X64_F8F6F4 with both operands in E2M1 runs at twice the int8 rate and its
// operands take 4 bits per value.  Every packed bit becomes the code 0x0 (0.0) or 0x1 (0.5), both
// operands carry the block scale 2 (E8M0 code 128), so a product of two set bits is exactly 1.0
// and the fp32 accumulator holds S, the count of positions where both are +1, exactly (K < 2^24).
// The element order inside a lane's 32 values is the same for both operands, which is all a dot
// product needs.  Same tile and staging as the int8 kernel; an LDS row is 32 bytes (+16 pad).
typedef int v8i_f4 __attribute__((ext_vector_type(8)));
typedef float v16f_f4 __attribute__((ext_vector_type(16)));
constexpr int F4_RS = 48;  // bytes per LDS row: 16-byte reads of 8 consecutive rows cover all banks

__device__ __forceinline__ uint32_t spread8_to_nibbles(uint32_t x) {
  // bits 0..7 of x -> bit 4*i of the result (three shift-or-mask steps)
  uint32_t y = (x | (x << 12)) & 0x000F000Fu;
  y = (y | (y << 6)) & 0x03030303u;
  y = (y | (y << 3)) & 0x11111111u;
  return y;
}

__device__ __forceinline__ void expand_store_fp4(uint64_t word, uint8_t *dst) {
  // 64 values -> 32 bytes
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    const uint32_t src = (uint32_t)(word >> (32 * g));
    v4i v;
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = (int)spread8_to_nibbles((src >> (8 * e)) & 0xFFu);
    *reinterpret_cast<v4i *>(dst + g * 16) = v;
  }
}

// Same workgroup shape as the int8 kernel: 2 x 2 waves of 64 x 64 outputs, one tile row per
// thread.  (A 256 x 256 tile with 16 waves, which halves the expansion per multiply-add, measured
// slower: 1616 against 1776 TBOPS on the 256 x 200704 x 2304 problem.)
__global__ __launch_bounds__(256, 2) void xnor_gemm_mfma_fp4_kernel(MfmaParams p) {
  constexpr int BM = MF_BM, BN = MF_BN;
  __shared__ __attribute__((aligned(16))) uint8_t sT[2][(BM + BN) * F4_RS];
  __shared__ int sPop[BM + BN];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int mi = blockIdx.x % p.tilesM, ni = blockIdx.x / p.tilesM;
  const int m0 = mi * BM, n0 = ni * BN;

  const int trow = tid;  // this thread's row of the tile: A rows first, then B rows
  const bool isA = trow < BM;
  const int grow = isA ? m0 + trow : n0 + (trow - BM);
  const bool row_ok = isA ? grow < p.M : grow < p.N;
  const uint64_t *rowp = isA ? p.A + (int64_t)grow * p.lda : p.B + (int64_t)grow * p.ldb;
  const int tail = p.K & 63;
  const uint64_t tail_mask = tail ? ((1ull << tail) - 1ull) : ~0ull;
  auto load_word = [&](int c) -> uint64_t {
    uint64_t w = 0;
    if (row_ok && c < p.Kw) {
      w = rowp[c];
      if (c == p.Kw - 1) w &= tail_mask;
    }
    return w;
  };
  auto expand_store = [&](uint64_t word, uint8_t *row_dst) { expand_store_fp4(word, row_dst); };

  v16f_f4 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;

  int pop = 0;
  uint64_t cur = load_word(0);
  pop += __popcll(cur);
  expand_store(cur, &sT[0][trow * F4_RS]);
  __syncthreads();

  // lane l: row l % 32 of a block, values 32 * (l / 32) .. + 31 of the 64-value chunk (16 bytes)
  const int arow = (64 * wm + (lane & 31)) * F4_RS + 16 * (lane >> 5);
  const int brow = (BM + 64 * wn + (lane & 31)) * F4_RS + 16 * (lane >> 5);
  const int scale2 = (int)0x80808080u;  // E8M0 128 = 2^1 in every byte

  for (int c = 0; c < p.Kw; ++c) {
    const int buf = c & 1;
    const bool more = c + 1 < p.Kw;
    uint64_t nxt = 0;
    if (more) nxt = load_word(c + 1);
    const uint8_t *T = sT[buf];
    v8i_f4 a[2], b[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
      const v4i t = *reinterpret_cast<const v4i *>(T + arow + mb * 32 * F4_RS);
      a[mb] = v8i_f4{t[0], t[1], t[2], t[3], 0, 0, 0, 0};
    }
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const v4i t = *reinterpret_cast<const v4i *>(T + brow + nb * 32 * F4_RS);
      b[nb] = v8i_f4{t[0], t[1], t[2], t[3], 0, 0, 0, 0};
    }
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
        acc[mb][nb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[mb], b[nb], acc[mb][nb], 4, 4, 0, scale2, 0,
                                                                      scale2);
    if (more) {
      pop += __popcll(nxt);
      expand_store(nxt, &sT[buf ^ 1][trow * F4_RS]);  // last read two iterations ago, before the previous barrier
      __syncthreads();
    }
  }

  sPop[tid] = pop;
  __syncthreads();
  auto row_pop = [&](int r) { return sPop[r]; };  // +1 count of tile row r (A rows first, then B rows)

#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const int nl = 64 * wn + 32 * nb + (lane & 31);
      const int n = n0 + nl;
      if (n >= p.N) continue;
      const int pb = row_pop(BM + nl);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int ml = 64 * wm + 32 * mb + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        const int m = m0 + ml;
        if (m < p.M) p.C[(int64_t)m * p.ldc + n] = p.K - 2 * (row_pop(ml) + pb) + 4 * (int)acc[mb][nb][r];
      }
    }
}

// ---- third form: operands kept expanded in memory ---------------------------------------------
// Both forms above spend most of their time expanding bits.  Here the expansion is a separate
// streaming pass (a layer's epilogue could write this format itself): a row of K binary values is
// stored as K E2M1 codes, +1.0 (0x2) or -1.0 (0xA), value k in nibble k % 2 of byte k / 2, padded
// with 0.0 (0x0) to a multiple of 64 values, i.e. 4 bits per value.  The matrix instruction then
// computes sum_k a_k * b_k directly: the result itself, exact in fp32 for K < 2^24, with no
// popcount correction, and the pad values contribute nothing.
//
// Workgroup: 4 waves as 2 x 2, each wave WTM x WTN blocks of 32 x 32 (2 x 2, 4 x 2 or 2 x 4; with
// 4 x 4 the accumulators alone fill the register file and the compiler spills); K consumed KCH
// values at a time through double-buffered LDS.  A chunk of a row is KCH / 2 bytes, stored with 16 bytes of
// padding, so that the 16-byte reads of eight consecutive rows cover all banks.
struct Fp4xParams {
  const uint8_t *A, *B;
  int64_t lda, ldb, ldc;  // lda, ldb in bytes
  int32_t *C;
  int M, N;
  int pieces;  // 16-byte pieces per row: 2 * ceil(K / 64)
  int tilesM;
  // convolution form (CONV = 1): B is a 4-bit NHWC image [Nimg, H, W, C / 2 bytes], column n is
  // output pixel n, piece j of its row is channels 32 * (j % ppt) .. + 31 of tap j / ppt, and the
  // output is NCHW (row m = output channel)
  int H, W, OH, OW, kW, sH, sW, pH, pW;
  int ppt;               // 16-byte pieces per tap: C / 32
  int64_t pix_bytes;     // C / 2
  int64_t img_stride;    // D * OH * OW outputs per image
  uint32_t OHW;
  FastDiv divPpt, divKW, divOW, divOH, divOHW;
};

template <int WTM, int WTN, int KCH, int CONV>
__global__ __launch_bounds__(256, (WTM * WTN <= 8) ? 2 : 1) void xnor_gemm_mfma_fp4x_kernel(Fp4xParams p) {
  constexpr int BM = 64 * WTM, BN = 64 * WTN, ROWS = BM + BN;
  constexpr int RS = KCH / 2 + 16;        // bytes per LDS row
  constexpr int PPR = KCH / 32;           // 16-byte pieces per row per chunk
  constexpr int PPT = ROWS * PPR / 256;   // pieces per thread per chunk
  static_assert(ROWS * PPR % 256 == 0, "staging must divide evenly");
  static_assert(2 * ROWS * RS <= 65536, "LDS budget");
  __shared__ __attribute__((aligned(16))) uint8_t sT[2][ROWS * RS];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int mi = blockIdx.x % p.tilesM, ni = blockIdx.x / p.tilesM;
  const int m0 = mi * BM, n0 = ni * BN;

  // this thread's pieces of a chunk: tile row (A rows first, then B rows) and piece within the chunk
  const uint8_t *gp[PPT];
  bool gok[PPT];
  int gq[PPT], soff[PPT];
  // convolution form, B rows: the pixel under tap (0, 0) of this thread's output pixel
  bool gconv[PPT];
  int gih0[PPT], giw0[PPT];
#pragma unroll
  for (int t = 0; t < PPT; ++t) {
    const int idx = t * 256 + tid;
    const int row = idx / PPR, q = idx % PPR;
    const bool isA = row < BM;
    const int grow = isA ? m0 + row : n0 + (row - BM);
    gok[t] = isA ? grow < p.M : grow < p.N;
    gq[t] = q;
    soff[t] = row * RS + 16 * q;
    gconv[t] = CONV && !isA;
    gih0[t] = giw0[t] = 0;
    if (CONV && !isA) {
      const uint32_t n = gok[t] ? (uint32_t)grow : 0u;
      const uint32_t tq = fdiv(n, p.divOW);
      const uint32_t ow = n - tq * (uint32_t)p.OW;
      const uint32_t img = fdiv(tq, p.divOH);
      const uint32_t oh = tq - img * (uint32_t)p.OH;
      gih0[t] = (int)oh * p.sH - p.pH;
      giw0[t] = (int)ow * p.sW - p.pW;
      gp[t] = p.B + (int64_t)img * p.H * p.W * p.pix_bytes;  // the pixel's image
    } else {
      gp[t] = (isA ? p.A + (int64_t)grow * p.lda : p.B + (int64_t)grow * p.ldb) + 16 * q;
    }
  }
  const int nchunks = (p.pieces + PPR - 1) / PPR;
  // Chunk c + 2 is requested before chunk c is multiplied and written to LDS after chunk c + 1's
  // multiplications have been issued: a chunk is only 2 * WTM * WTN matrix instructions per wave,
  // far less than a memory round trip, so one chunk of distance leaves every chunk waiting for
  // its loads.  Two register sets, used alternately (the loop body is written out for both).
  v4i stage0[PPT], stage1[PPT];
  auto stage_load = [&](int c, v4i(&st)[PPT]) {
#pragma unroll
    for (int t = 0; t < PPT; ++t) {
      v4i v = {0, 0, 0, 0};  // rows past M / N and pieces past the row's end: 0.0, adds nothing
      const int j = c * PPR + gq[t];
      if (gok[t] && j < p.pieces) {
        if (CONV && gconv[t]) {
          const uint32_t tap = fdiv((uint32_t)j, p.divPpt);
          const uint32_t cq = (uint32_t)j - tap * (uint32_t)p.ppt;
          const uint32_t kh = fdiv(tap, p.divKW);
          const int ih = gih0[t] + (int)kh, iw = giw0[t] + (int)(tap - kh * (uint32_t)p.kW);
          if (ih >= 0 && ih < p.H && iw >= 0 && iw < p.W)
            v = *reinterpret_cast<const v4i *>(gp[t] + ((int64_t)ih * p.W + iw) * p.pix_bytes + 16 * (int64_t)cq);
          else
            v = v4i{0x22222222, 0x22222222, 0x22222222, 0x22222222};  // taps outside the image: +1.0
        } else {
          v = *reinterpret_cast<const v4i *>(gp[t] + (int64_t)c * (KCH / 2));
        }
      }
      st[t] = v;
    }
  };
  auto stage_store = [&](int buf, const v4i(&st)[PPT]) {
#pragma unroll
    for (int t = 0; t < PPT; ++t) *reinterpret_cast<v4i *>(&sT[buf][soff[t]]) = st[t];
  };

  v16f_f4 acc[WTM][WTN];
#pragma unroll
  for (int a = 0; a < WTM; ++a)
#pragma unroll
    for (int b = 0; b < WTN; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;

  // lane l: row l % 32 of a block, values 32 * (l / 32) .. + 31 of a 64-value step (16 bytes)
  const int arow = (32 * WTM * wm + (lane & 31)) * RS + 16 * (lane >> 5);
  const int brow = (BM + 32 * WTN * wn + (lane & 31)) * RS + 16 * (lane >> 5);
  const int scale1 = (int)0x7F7F7F7Fu;  // E8M0 127 = 2^0 in every byte

  auto multiply = [&](int buf) {
    const uint8_t *T = sT[buf];
#pragma unroll
    for (int ks = 0; ks < KCH / 64; ++ks) {
      v8i_f4 a[WTM], b[WTN];
#pragma unroll
      for (int mb = 0; mb < WTM; ++mb) {
        const v4i t = *reinterpret_cast<const v4i *>(T + arow + mb * 32 * RS + ks * 32);
        a[mb] = v8i_f4{t[0], t[1], t[2], t[3], 0, 0, 0, 0};
      }
#pragma unroll
      for (int nb = 0; nb < WTN; ++nb) {
        const v4i t = *reinterpret_cast<const v4i *>(T + brow + nb * 32 * RS + ks * 32);
        b[nb] = v8i_f4{t[0], t[1], t[2], t[3], 0, 0, 0, 0};
      }
#pragma unroll
      for (int mb = 0; mb < WTM; ++mb)
#pragma unroll
        for (int nb = 0; nb < WTN; ++nb)
          acc[mb][nb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[mb], b[nb], acc[mb][nb], 4, 4, 0, scale1, 0,
                                                                        scale1);
    }
  };

  // chunk 0 -> LDS buffer 0; chunk 1 waits in register set 1
  stage_load(0, stage0);
  stage_store(0, stage0);
  if (nchunks > 1) stage_load(1, stage1);
  __syncthreads();
  // Chunk c sits in LDS buffer c % 2 and chunk c + 1 in register set (c + 1) % 2.  The other
  // LDS buffer was last read in chunk c - 1, before the previous barrier.
  for (int c = 0; c < nchunks; c += 2) {
    if (c + 2 < nchunks) stage_load(c + 2, stage0);
    multiply(0);
    if (c + 1 < nchunks) {
      stage_store(1, stage1);
      __syncthreads();
      if (c + 3 < nchunks) stage_load(c + 3, stage1);
      multiply(1);
      if (c + 2 < nchunks) {
        stage_store(0, stage0);
        __syncthreads();
      }
    }
  }

  // D[i][j] of a 32x32 block: lane l holds column j = l % 32; register r holds row
  // i = 8*(r/4) + 4*(l/32) + (r%4).
#pragma unroll
  for (int mb = 0; mb < WTM; ++mb)
#pragma unroll
    for (int nb = 0; nb < WTN; ++nb) {
      const int n = n0 + 32 * WTN * wn + 32 * nb + (lane & 31);
      if (n >= p.N) continue;
      int64_t col = n;  // row-major C; NCHW: image * (D * OH * OW) + pixel, rows OH * OW apart
      if (CONV) {
        const uint32_t img = fdiv((uint32_t)n, p.divOHW);
        col = (int64_t)img * p.img_stride + ((uint32_t)n - img * p.OHW);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + 32 * WTM * wm + 32 * mb + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (m < p.M) __builtin_nontemporal_store((int)acc[mb][nb][r], p.C + (int64_t)m * p.ldc + col);
      }
    }
}

// Packed sign rows -> E2M1 rows: one thread per 64-bit word (32 bytes out).
__global__ __launch_bounds__(256) void expand_fp4_kernel(const uint64_t *__restrict__ src, int64_t src_ld, int K, int Kw,
                                                         uint8_t *__restrict__ dst, int64_t dst_ld, int64_t total) {
  const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (g >= total) return;
  const int64_t row = g / Kw;
  const int cw = (int)(g - row * Kw);
  const uint64_t word = src[row * src_ld + cw];
  const int left = K - 64 * cw;  // values of this word that exist: 1..64 (or more)
  const uint64_t vmask = left >= 64 ? ~0ull : ((1ull << left) - 1ull);
  uint8_t *o = dst + row * dst_ld + 32 * (int64_t)cw;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint32_t bits = (uint32_t)(word >> (32 * h)), val = (uint32_t)(vmask >> (32 * h));
    v4i v;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t y = spread8_to_nibbles((bits >> (8 * e)) & 0xFFu);  // bit 4i = value i is +1
      const uint32_t m = spread8_to_nibbles((val >> (8 * e)) & 0xFFu);   // bit 4i = value i exists
      // -1.0 is 0xA, +1.0 is 0x2: clear the sign bit where the value is +1; 0x0 where there is no value
      v[e] = (int)((0xAAAAAAAAu ^ (y << 3)) & (m * 0xFu));
    }
    *reinterpret_cast<v4i *>(o + 16 * h) = v;
  }
}

template <int WTM, int WTN, int KCH, int CONV>
static void launch_fp4x(const Fp4xParams &p0, int64_t M, int64_t N, hipStream_t s) {
  Fp4xParams p = p0;
  constexpr int BM = 64 * WTM, BN = 64 * WTN;
  p.tilesM = (int)((M + BM - 1) / BM);
  const int64_t blocks = (int64_t)p.tilesM * ((N + BN - 1) / BN);
  hipLaunchKernelGGL((xnor_gemm_mfma_fp4x_kernel<WTM, WTN, KCH, CONV>), dim3((unsigned)blocks), dim3(256), 0, s, p);
}

static bnn_status mfma_ablation_common(const uint64_t *A, int64_t lda, const uint64_t *B, int64_t ldb, int32_t *C,
                                       int64_t ldc, int64_t M, int64_t N, int64_t K, void *stream, bool fp4) {
  if (M < 0 || N < 0 || K <= 0) return BNN_ERR_SHAPE;
  const int64_t Kw = bnn_packed_words(K);
  if (lda < Kw || ldb < Kw || ldc < N) return BNN_ERR_STRIDE;
  if (M == 0 || N == 0) return BNN_OK;
  if (!A || !B || !C) return BNN_ERR_NULL;
  if (!aligned16(A) || !aligned16(B) || !aligned16(C)) return BNN_ERR_ALIGN;
  // the fp4 form counts in fp32: exact below 2^24
  if (M > 0x7fffff00LL || N > 0x7fffff00LL || K > (fp4 ? 0xffffffLL : 0x1fffffffLL)) return BNN_ERR_UNSUPPORTED;
  MfmaParams p;
  p.A = A; p.B = B; p.lda = lda; p.ldb = ldb; p.ldc = ldc; p.C = C;
  p.M = (int)M; p.N = (int)N; p.K = (int)K; p.Kw = (int)Kw;
  p.tilesM = (int)((M + MF_BM - 1) / MF_BM);
  const int64_t blocks = (int64_t)p.tilesM * ((N + MF_BN - 1) / MF_BN);
  if (blocks > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  {
    ProfScope ps(fp4 ? KID_XNOR_GEMM_MFMA_FP4 : KID_XNOR_GEMM_MFMA, s);
    if (fp4)
      hipLaunchKernelGGL(xnor_gemm_mfma_fp4_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p);
    else
      hipLaunchKernelGGL(xnor_gemm_mfma_i8_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p);
  }
  return launch_status();
}

}  // namespace bnn

using namespace bnn;

extern "C" bnn_status bnn_xnor_gemm_mfma_fp4(const uint64_t *A, int64_t lda, const uint64_t *B, int64_t ldb, int32_t *C,
                                             int64_t ldc, int64_t M, int64_t N, int64_t K, void *stream) {
  return mfma_ablation_common(A, lda, B, ldb, C, ldc, M, N, K, stream, true);
}

extern "C" int64_t bnn_fp4_row_bytes(int64_t K) { return K <= 0 ? 0 : 32 * bnn_packed_words(K); }

extern "C" bnn_status bnn_expand_fp4(const uint64_t *src, int64_t rows, int64_t K, int64_t src_ld, uint8_t *dst,
                                     int64_t dst_ld_bytes, void *stream) {
  if (rows < 0 || K <= 0) return BNN_ERR_SHAPE;
  const int64_t Kw = bnn_packed_words(K);
  if (src_ld < Kw || dst_ld_bytes < 32 * Kw || (dst_ld_bytes & 15)) return BNN_ERR_STRIDE;
  if (rows == 0) return BNN_OK;
  if (!src || !dst) return BNN_ERR_NULL;
  if (!aligned16(src) || !aligned16(dst)) return BNN_ERR_ALIGN;
  if (K > 0xffffffLL || rows > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  const int64_t total = rows * Kw, blocks = (total + 255) / 256;
  if (blocks > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  {
    ProfScope ps(KID_EXPAND_FP4, s);
    hipLaunchKernelGGL(expand_fp4_kernel, dim3((unsigned)blocks), dim3(256), 0, s, src, src_ld, (int)K, (int)Kw, dst,
                       dst_ld_bytes, total);
  }
  return launch_status();
}

// tile: -1 chosen here; 0 128 x 128; 1 256 x 128; 2 128 x 256
static bnn_status fp4x_impl(const uint8_t *A4, int64_t lda_bytes, const uint8_t *B4, int64_t ldb_bytes, int32_t *C,
                            int64_t ldc, int64_t M, int64_t N, int64_t K, int tile, void *stream) {
  if (M < 0 || N < 0 || K <= 0) return BNN_ERR_SHAPE;
  const int64_t rb = bnn_fp4_row_bytes(K);
  if (lda_bytes < rb || ldb_bytes < rb || (lda_bytes & 15) || (ldb_bytes & 15) || ldc < N) return BNN_ERR_STRIDE;
  if (tile < -1 || tile > 2) return BNN_ERR_SHAPE;
  if (M == 0 || N == 0) return BNN_OK;
  if (!A4 || !B4 || !C) return BNN_ERR_NULL;
  if (!aligned16(A4) || !aligned16(B4) || !aligned16(C)) return BNN_ERR_ALIGN;
  if (M > 0x7fffff00LL || N > 0x7fffff00LL || K > 0xffffffLL) return BNN_ERR_UNSUPPORTED;  // fp32 counts: exact below 2^24
  if (((M + 127) / 128) * ((N + 127) / 128) > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  Fp4xParams p = {};
  p.A = A4; p.B = B4; p.lda = lda_bytes; p.ldb = ldb_bytes; p.ldc = ldc; p.C = C;
  p.M = (int)M; p.N = (int)N; p.pieces = (int)(rb / 16); p.tilesM = 0;
  hipStream_t s = (hipStream_t)stream;
  {
    ProfScope ps(KID_XNOR_GEMM_MFMA_FP4X, s);
    if (tile < 0) {
      // the larger tile along the longer side when it still gives every compute unit two workgroups
      // (measured: 256 x 200704 x 2304 100 us on 256 x 128 tiles against 111; 128 x 131072 x 1152
      // 24.5 us on 128 x 256 against 28.4; 512 x 16384 x 4608 33 us on 128 x 128 against 39.5)
      const int64_t two_per_cu = 2 * (int64_t)device_cu_count();
      if (M <= 128) tile = (N + 255) / 256 >= two_per_cu ? 2 : 0;
      else tile = ((M + 255) / 256) * ((N + 127) / 128) >= two_per_cu ? 1 : 0;
    }
    if (tile == 0) launch_fp4x<2, 2, 128, 0>(p, M, N, s);
    else if (tile == 1) launch_fp4x<4, 2, 128, 0>(p, M, N, s);
    else launch_fp4x<2, 4, 128, 0>(p, M, N, s);
  }
  return launch_status();
}

extern "C" bnn_status bnn_xnor_gemm_mfma_fp4_expanded(const uint8_t *A4, int64_t lda_bytes, const uint8_t *B4,
                                                      int64_t ldb_bytes, int32_t *C, int64_t ldc, int64_t M, int64_t N,
                                                      int64_t K, void *stream) {
  return fp4x_impl(A4, lda_bytes, B4, ldb_bytes, C, ldc, M, N, K, -1, stream);
}

extern "C" bnn_status bnn_conv2d_mfma_fp4_expanded(const uint8_t *x4, const uint8_t *w4, int N, int C, int H, int W,
                                                   int D, int kH, int kW, int sH, int sW, int pH, int pW,
                                                   int32_t *out_i32, void *stream) {
  bnn_status st = check_conv_geometry(N, C, H, W, kH, kW, sH, sW, pH, pW);
  if (st != BNN_OK) return st;
  if (D < 0) return BNN_ERR_SHAPE;
  if (C % 64 != 0) return BNN_ERR_UNSUPPORTED;  // whole words per pixel: no pad channels inside a tap
  if (N == 0 || D == 0) return BNN_OK;
  if (!x4 || !w4 || !out_i32) return BNN_ERR_NULL;
  if (!aligned16(x4) || !aligned16(w4) || !aligned16(out_i32)) return BNN_ERR_ALIGN;
  const int64_t OH = bnn_conv_out_dim(H, kH, sH, pH), OW = bnn_conv_out_dim(W, kW, sW, pW);
  const int64_t P = (int64_t)N * OH * OW, K = (int64_t)C * kH * kW;
  if (K > 0xffffffLL || P > 0x7fffff00LL || D > 0x7fffff00LL || (int64_t)D * P > 0x7fffffffLL * 8 ||
      ((D + 127) / 128) * ((P + 127) / 128) > 0x7fffffffLL)
    return BNN_ERR_UNSUPPORTED;
  Fp4xParams p = {};
  p.A = w4; p.B = x4; p.lda = K / 2; p.ldb = 0; p.ldc = OH * OW; p.C = out_i32;
  p.M = D; p.N = (int)P; p.pieces = (int)(K / 32); p.tilesM = 0;
  p.H = H; p.W = W; p.OH = (int)OH; p.OW = (int)OW; p.kW = kW; p.sH = sH; p.sW = sW; p.pH = pH; p.pW = pW;
  p.ppt = C / 32;
  p.pix_bytes = C / 2;
  p.img_stride = (int64_t)D * OH * OW;
  p.OHW = (uint32_t)(OH * OW);
  p.divPpt = FastDiv((uint32_t)p.ppt);
  p.divKW = FastDiv((uint32_t)kW);
  p.divOW = FastDiv((uint32_t)OW);
  p.divOH = FastDiv((uint32_t)OH);
  p.divOHW = FastDiv(p.OHW);
  hipStream_t s = (hipStream_t)stream;
  {
    ProfScope ps(KID_XNOR_GEMM_MFMA_FP4X, s);
    // 128 x 128 tiles: with the gather's addressing the larger ones no longer fit the register file
    // (measured with spills: cfg 5a 142 / 179 us against 108)
    launch_fp4x<2, 2, 128, 1>(p, D, P, s);
  }
  return launch_status();
}

// Declared in bnn_testing.h.
extern "C" bnn_status bnn_testing_xnor_gemm_mfma_fp4_expanded(const uint8_t *A4, int64_t lda_bytes, const uint8_t *B4,
                                                              int64_t ldb_bytes, int32_t *C, int64_t ldc, int64_t M,
                                                              int64_t N, int64_t K, int tile, void *stream) {
  return fp4x_impl(A4, lda_bytes, B4, ldb_bytes, C, ldc, M, N, K, tile, stream);
}

extern "C" bnn_status bnn_xnor_gemm_mfma_i8(const uint64_t *A, int64_t lda, const uint64_t *B, int64_t ldb, int32_t *C,
                                            int64_t ldc, int64_t M, int64_t N, int64_t K, void *stream) {
  return mfma_ablation_common(A, lda, B, ldb, C, ldc, M, N, K, stream, false);
}
