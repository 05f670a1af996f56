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

extern "C" bnn_status bnn_xnor_gemm_mfma_i8(const uint64_t *A, int64_t lda, const uint64_t *B, int64_t ldb, int32_t *C,
                                            int64_t ldc, int64_t M, int64_t N, int64_t K, void *stream) {
  return mfma_ablation_common(A, lda, B, ldb, C, ldc, M, N, K, stream, false);
}
