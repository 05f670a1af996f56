// Xnor-Bitcount GEMM (section 3.2 of the paper) for gfx950, in the exclusive-or form
//     C[m,n] = K - 2 * sum_w popcount(A[m,w] ^ B[n,w]).
//
// CDNA4 has no 1-bit matrix instruction, so the contraction runs on the vector ALU:
// two lane-instructions per 32 bit-MACs per output (v_xor_b32, then v_bcnt_u32_b32
// which adds its popcount into the accumulator).  The kernel is built so that the
// inner loop is almost nothing else:
//   * lanes of a wave run along N (64 consecutive columns per register column);
//     every lane keeps TM x TN int32 accumulators;
//   * the TM rows of A a wave works on are the same for all of its lanes, so A is
//     fetched with SCALAR loads into SGPRs and enters v_xor as the scalar operand:
//     no LDS traffic, no VGPRs and no VALU instructions are spent on A;
//   * the block's B tile (BN columns x KC dwords) is staged once per K-chunk through
//     LDS, row-per-column with a 4-dword pad so that both the 16-byte staging writes
//     and the 16-byte per-lane reads are bank-conflict free; the next chunk's global
//     loads are in flight while the current chunk is computed;
//   * full chunks run a fully unrolled mask-free path; only the final partial chunk
//     (K not a multiple of 32*KC) takes a per-dword path that masks the bits past K;
//   * K - 2*acc, the optional fma(scale, acc, bias) and the NCHW scatter of a
//     convolution happen once in the store, 256 contiguous bytes per wave store.
// Workgroup ids are remapped so that tiles sharing a B tile run on the same XCD
// (one L2 per XCD; hardware deals consecutive ids round-robin over the 8 XCDs).
#include "common.h"

namespace bnn {

using u32x4 = uint32_t __attribute__((ext_vector_type(4)));
typedef u32x4 u32x4_a8 __attribute__((aligned(8)));
// A is only ever read by the kernel.  Reading it through the constant address space lets
// the compiler use scalar (SMEM) loads for the wave-uniform addresses even after a barrier.
#define BNN_CONST_AS __attribute__((address_space(4)))
typedef const uint32_t BNN_CONST_AS *cu32_ptr;
typedef const u32x4_a8 BNN_CONST_AS *cu32x4_ptr;

// acc += popcount(x) as ONE instruction.  Written as asm because the optimizer otherwise
// re-associates a chain of popcount-adds into v_bcnt(x, 0) plus separate three-operand adds,
// which costs 25 % more VALU instructions in the inner loop.
__device__ __forceinline__ int popc_acc(uint32_t x, int acc) {
  asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc) : "v"(x));
  return acc;
}

template <int TM, int TN, int WM, int WN, int KC>
struct GemmCfg {
  static constexpr int BM = TM * WM;
  static constexpr int BN = 64 * TN * WN;
  static constexpr int THREADS = 64 * WM * WN;
  static constexpr int RS = KC + 4;                      // LDS row stride in dwords
  static constexpr int PIECES = BN * (KC / 4);           // 16-byte pieces per chunk
  static constexpr int PPT = (PIECES + THREADS - 1) / THREADS;
  static_assert(KC % 4 == 0, "chunk must be whole 16-byte pieces");
  static_assert(PIECES % THREADS == 0, "staging must divide evenly");
};

template <int TM, int TN, int WM, int WN, int KC, int MINB>
__global__ __launch_bounds__(64 * WM * WN, MINB) void xnor_gemm_kernel(GemmParams p) {
  using Cfg = GemmCfg<TM, TN, WM, WN, KC>;
  constexpr int RS = Cfg::RS;
  constexpr int PPT = Cfg::PPT;
  constexpr int QPR = KC / 4;  // pieces per row
  __shared__ __attribute__((aligned(16))) uint32_t sB[Cfg::BN * RS];

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

  // Dword offsets of this wave's TM rows (clamped: rows past M recompute row M-1 and are
  // not stored).  32-bit: the host checks that M * lda32 < 2^32.
  uint32_t aoff[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    int m = m0 + i;
    m = m < p.M ? m : p.M - 1;
    aoff[i] = (uint32_t)m * (uint32_t)p.lda32;
  }

  const cu32_ptr Ac = (cu32_ptr)(uintptr_t)p.A;

  int acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = 0;

  const int nchunks = (p.Kd + KC - 1) / KC;
  const int full_chunks = p.Kbits / (32 * KC);  // chunks whose every bit takes part
  const int last_w = p.Kw64 - 1;
  const int tail_bits = p.Kbits & 63;
  const uint64_t tail_mask = tail_bits ? ((1ull << tail_bits) - 1ull) : ~0ull;

  // ---- staging: global -> registers -> LDS --------------------------------------
  u32x4 stage[PPT];
  auto stage_load = [&](int chunk) {
#pragma unroll
    for (int t = 0; t < PPT; ++t) {
      const int idx = t * Cfg::THREADS + tid;
      const int row = idx / QPR, q = idx % QPR;
      const int n = n0 + row;
      const int w0 = chunk * (KC / 2) + 2 * q;
      u32x4 v = {0u, 0u, 0u, 0u};
      if (n < p.N && w0 <= last_w) {
        const uint64_t *src = p.B + (int64_t)n * p.ldb + w0;
        uint64_t x0, x1 = 0;
        if (p.b_vec16 && w0 + 1 <= last_w) {
          const u32x4 raw = *reinterpret_cast<const u32x4 *>(src);
          x0 = ((uint64_t)raw.y << 32) | raw.x;
          x1 = ((uint64_t)raw.w << 32) | raw.z;
        } else {
          x0 = src[0];
          if (w0 + 1 <= last_w) x1 = src[1];
        }
        if (w0 == last_w) x0 &= tail_mask;
        if (w0 + 1 == last_w) x1 &= tail_mask;
        v.x = (uint32_t)x0; v.y = (uint32_t)(x0 >> 32); v.z = (uint32_t)x1; v.w = (uint32_t)(x1 >> 32);
      }
      stage[t] = v;
    }
  };
  auto stage_store = [&]() {
#pragma unroll
    for (int t = 0; t < PPT; ++t) {
      const int idx = t * Cfg::THREADS + tid;
      const int row = idx / QPR, q = idx % QPR;
      *reinterpret_cast<u32x4 *>(&sB[row * RS + q * 4]) = stage[t];
    }
  };

  const uint32_t *sBlane = &sB[(wn * 64 * TN + lane) * RS];

  stage_load(0);
  for (int c = 0; c < nchunks; ++c) {
    if (c > 0) __syncthreads();  // everyone is done reading the previous chunk
    stage_store();
    __syncthreads();
    if (c + 1 < nchunks) stage_load(c + 1);

    const int kd0 = c * KC;
    const cu32_ptr Ak = Ac + kd0;  // wave-uniform
    // one sub-step: 4 dwords of every row against 4 dwords of every column, no masks
    auto substep = [&](int s) {
      u32x4 b[TN];
#pragma unroll
      for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const u32x4 *>(&sBlane[j * 64 * RS + s]);
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const u32x4 a = *(cu32x4_ptr)(Ak + aoff[i] + s);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          acc[i][j] = popc_acc(a.x ^ b[j].x, acc[i][j]);
          acc[i][j] = popc_acc(a.y ^ b[j].y, acc[i][j]);
          acc[i][j] = popc_acc(a.z ^ b[j].z, acc[i][j]);
          acc[i][j] = popc_acc(a.w ^ b[j].w, acc[i][j]);
        }
      }
    };
    if (c < full_chunks) {
#pragma unroll
      for (int s = 0; s < KC; s += 4) substep(s);
    } else {
      // final partial chunk: whole mask-free sub-steps first, then one dword at a time.
      // B is already masked / zero-filled by the staging; A is masked here.
      const int kd_end = p.Kd < kd0 + KC ? p.Kd : kd0 + KC;  // dwords holding any bit
      const int kd_full = p.Kbits >> 5;                       // dwords holding 32 bits
      int s = 0;
#pragma unroll 1
      for (; kd0 + s + 4 <= kd_full; s += 4) substep(s);
      const int tb32 = p.Kbits & 31;
#pragma unroll 1
      for (int kd = kd0 + s; kd < kd_end; ++kd) {
        const uint32_t amask = (kd == p.Kd - 1 && tb32) ? ((1u << tb32) - 1u) : 0xffffffffu;
        uint32_t b[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) b[j] = sBlane[j * 64 * RS + (kd - kd0)];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          const uint32_t a = Ac[aoff[i] + kd] & amask;
#pragma unroll
          for (int j = 0; j < TN; ++j) acc[i][j] = popc_acc(a ^ b[j], acc[i][j]);
        }
      }
    }
  }

  // ---- store ------------------------------------------------------------------------
  // The store-only parameters are re-read from the kernel-argument segment here, through a
  // pointer the optimizer cannot see through, so that they do not occupy SGPRs (or spill
  // slots) during the main loop.
  const GemmParams BNN_CONST_AS *kp = (const GemmParams BNN_CONST_AS *)__builtin_amdgcn_kernarg_segment_ptr();
  asm volatile("" : "+s"(kp));
  const int M = kp->M, N = kp->N, Kformula = kp->Kformula, axis = kp->axis;
  int32_t *const Cp = kp->C;
  float *const Yp = kp->Y;
  const float *const scale = kp->scale, *const bias = kp->bias;
  const int64_t ldc = kp->ldc, ldy = kp->ldy, img_stride = kp->img_stride;
  const uint32_t OHW = kp->OHW;
  FastDiv divOHW;
  divOHW.d = kp->divOHW.d; divOHW.mul = kp->divOHW.mul; divOHW.shift = kp->divOHW.shift;

  const int nbase = n0 + wn * 64 * TN + lane;
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
        if (cp) *cp = v;
        if (yp) {
          if (axis == BNN_CH_ROW) {
            sc = scale[m0 + i];
            bi = bias[m0 + i];
          }
          *yp = fmaf(sc, (float)v, bi);
        }
      }
      if (cp) cp += ldc;
      if (yp) yp += ldy;
    }
  }
}

// ---- host side ----------------------------------------------------------------------
template <int TM, int TN, int WM, int WN, int KC, int MINB>
static bnn_status launch_cfg(GemmParams &p, hipStream_t s, int kid) {
  using Cfg = GemmCfg<TM, TN, WM, WN, KC>;
  p.tilesM = (p.M + Cfg::BM - 1) / Cfg::BM;
  p.tilesN = (p.N + Cfg::BN - 1) / Cfg::BN;
  const int64_t blocks = (int64_t)p.tilesM * p.tilesN;
  if (blocks > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  ProfScope ps(kid, s);
  hipLaunchKernelGGL((xnor_gemm_kernel<TM, TN, WM, WN, KC, MINB>), dim3((unsigned)blocks), dim3(Cfg::THREADS), 0, s,
                     p);
  return launch_status();
}

int g_force_cfg = -1;  // test / tuning hook: -1 = heuristic

// Tile choice: the large tile (64 x 512) has the best ratio of VALU work to everything
// else but needs enough tiles to fill 256 CUs twice over; smaller problems fall back to
// finer tiles so that every CU has work.
bnn_status run_gemm(GemmParams &p, hipStream_t s) {
  const int64_t tilesL = (int64_t)((p.M + 63) / 64) * ((p.N + 511) / 512);
  const int64_t tilesMd = (int64_t)((p.M + 31) / 32) * ((p.N + 255) / 256);
  int cfg = g_force_cfg;
  if (cfg < 0) cfg = tilesL >= 512 ? 0 : (tilesMd >= 512 ? 1 : 2);
  switch (cfg) {
    case 0: return launch_cfg<8, 8, 8, 1, 8, 1>(p, s, KID_XNOR_GEMM);
    case 1: return launch_cfg<8, 4, 4, 1, 8, 2>(p, s, KID_XNOR_GEMM);
    default: return launch_cfg<8, 1, 4, 1, 16, 2>(p, s, KID_XNOR_GEMM_SMALL);
  }
}

static bnn_status gemm_common(const uint64_t *A, int64_t lda, const uint64_t *B, int64_t ldb, int64_t M, int64_t N,
                              int64_t K, int32_t *C, int64_t ldc, float *Y, int64_t ldy, const float *scale,
                              const float *bias, bnn_ch_axis axis, void *stream) {
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
  if (M > 0x7fffffffLL || N > 0x7ffffff0LL || K > 0x7fffffffLL) return BNN_ERR_UNSUPPORTED;
  if (M * 2 * lda > 0xffffffffLL) return BNN_ERR_UNSUPPORTED;  // 32-bit dword offsets into A
  GemmParams p;
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
  return run_gemm(p, (hipStream_t)stream);
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

// Tuning / test hook (not declared in the public header): force a tile configuration.
extern "C" void bnn_internal_force_gemm_cfg(int cfg) { g_force_cfg = cfg; }
