// Internal helpers shared by the translation units of libbnn (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bnn.h"

namespace bnn {

// Kernel ids reported by the timing hook.
enum KernelId : int {
  KID_ENCODE_ROWS = 0,
  KID_PACK_CONV_WEIGHT = 1,
  KID_ENCODE_NCHW = 2,
  KID_IM2COL_GATHER = 3,
  KID_XNOR_GEMM = 4,
  KID_MAXPOOL = 5,
  KID_CONV_F32 = 6,
  KID_FC_F32 = 7,
  KID_VALU_PROBE = 8,
  KID_COPY_PROBE = 9,
  KID_XNOR_GEMM_SMALL = 10,
  KID_CONV_F32_SIGN = 11,
  KID_XNOR_GEMM_MFMA = 12,
  KID_CONTROL_CONV_F32 = 13,
  KID_XNOR_GEMM_MFMA_FP4 = 14,
  KID_XNOR_GEMM_LOWK = 15,
  KID_XNOR_CONV_LATENCY = 16,
  KID_EXPAND_FP4 = 17,
  KID_XNOR_GEMM_MFMA_FP4X = 18,
  KID_COUNT = 19
};

// Timing hook: records an event pair around a launch when profiling is on.
void prof_begin(int kernel_id, hipStream_t s);
void prof_end(hipStream_t s);

struct ProfScope {
  hipStream_t s;
  ProfScope(int kid, hipStream_t st) : s(st) { prof_begin(kid, st); }
  ~ProfScope() { prof_end(s); }
};

inline bnn_status launch_status() {
  return hipGetLastError() == hipSuccess ? BNN_OK : BNN_ERR_HIP;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Division of a 32-bit unsigned value by a runtime constant with one mulhi and one
// shift (round-up method; exact for every n < 2^31 and 1 <= d < 2^31).
struct FastDiv {
  uint32_t d, mul, shift;
  __host__ __device__ FastDiv() : d(1), mul(0), shift(0) {}
  __host__ __device__ explicit FastDiv(uint32_t div) : d(div) {
    if (div == 1) {
      mul = 0;
      shift = 0;
      return;
    }
    uint32_t l = 0;
    while ((1ull << l) < div) ++l;  // l = ceil(log2 d)
    shift = l - 1;
    // m = floor(2^32 * (2^l - d) / d) + 1, used as q = (mulhi(n, m) + n) >> l, rewritten
    // below so that no 33-bit intermediate is needed for n < 2^31.
    mul = (uint32_t)(((1ull << 32) * ((1ull << l) - div)) / div + 1);
  }
};

__device__ __forceinline__ uint32_t fdiv(uint32_t n, const FastDiv &f) {
  if (f.d == 1) return n;
  uint32_t t = __umulhi(n, f.mul);
  return (t + ((n - t) >> 1)) >> f.shift;
}

// ---- cross-file internals ---------------------------------------------------------------
// Geometry of an implicit-GEMM B operand: column n of the GEMM is output pixel n of a
// convolution over a packed NHWC image (ceil(C/64) words per pixel), and word w of its
// row is word (w mod Cw) of tap (w div Cw), taps ordered (kh, kw).
struct ConvGeom {
  const uint64_t *act;  // [Nimg, H, W, Cw]
  int Nimg, C, H, W, Cw, OH, OW, kH, kW, sH, sW, pH, pW;
  int pool;             // 0, or 2: columns are ordered window-major (see decode_col in gemm.hip)
  FastDiv divCw, divKW;
  FastDiv divOW, divOH; // output dims, or pooled output dims when pool == 2
};

struct GemmParams {
  const uint32_t *A;   // [M, lda32] dwords
  const uint64_t *B;   // [N, ldb] words (explicit B only)
  int64_t lda32, ldb;
  int M, N;
  int Kd;              // dwords per row that hold bits of the reduction (ceil(Kbits/32))
  int Kbits;           // bits per row taking part in the exclusive-or
  int Kformula;        // K of the formula (true reduction length)
  int Kw64;            // words per row that may be read (ceil(Kbits/64))
  int b_vec16;         // B rows may be read with 16-byte loads
  int32_t *C;
  float *Y;
  int64_t ldc, ldy;    // row (m) strides of C and Y
  const float *scale, *bias;
  int axis;
  uint32_t OHW;        // columns per image; n -> (img, pix) = (n / OHW, n % OHW)
  FastDiv divOHW;
  int64_t img_stride;  // elements between images in C / Y
  int tilesM, tilesN;
  int prio_from;       // workgroups with id >= prio_from lower their wave priority as they advance through K
  int n_cu;            // compute units of the device (host only: launch heuristics)
  int nt_store;        // int32 / fp32 tile stores are line-aligned: use non-temporal stores
  int colperm;         // 256-column tiles, int32 / fp32 output: LDS row 64 * j + l holds tile column 4 * l + j,
                       // so a lane's four columns are consecutive and go out as one 16-byte store per row
  ConvGeom g;          // implicit B only
  uint64_t *outp;      // packed-sign output [pixels, cw_out] (packed epilogue only)
  int cw_out;
};

// Per-call choice of the GEMM variant.  The entry points of bnn.h always pass the defaults (size
// heuristic, table-driven gather where the geometry allows it); only the entry points of
// bnn_testing.h pass anything else.  Every variant computes the same values.
struct GemmTune {
  int cfg = -1;   // tile configuration (numbering in bnn_testing.h); -1 = heuristic
  int lean = 1;   // 0 = always the general implicit-GEMM gather
};

// Compute units of the current device (queried once per device, then cached).
int device_cu_count();

// Launch the exclusive-or / popcount GEMM described by p (tilesM / tilesN are filled in).
// bmode 0: B is an explicit [N, ldb] matrix; 1: B is gathered from p.g (implicit GEMM; the
// launcher switches to the lean gather, kernel mode 2, when the geometry allows it).
// emode 0: int32 / fp32 store; 1: packed sign(fma(scale, acc, bias)) store, optional 2x2 pool.
bnn_status run_gemm(GemmParams &p, int bmode, int emode, hipStream_t s, const GemmTune &tune = GemmTune());

// Short-row GEMM (gemm_lowk.hip): rows of two or four words, explicit B, 16-byte stores.
bool lowk_applicable(const GemmParams &p);
bnn_status launch_lowk(GemmParams &p, int groups, hipStream_t s);

// Latency form of the implicit-GEMM convolution (gemm_latency.hip): few output pixels, K split
// over ks (2 or 4) slices inside a workgroup.  emode as for run_gemm.
bool latency_applicable(const GemmParams &p);
bnn_status launch_latency(GemmParams &p, int emode, int ks, hipStream_t s);

// Conv helpers (im2col.hip).  check_conv_geometry validates shapes and 32-bit limits;
// run_im2col launches encode (+ gather) with already validated arguments.
bnn_status check_conv_geometry(int N, int C, int H, int W, int kH, int kW, int sH, int sW, int pH, int pW);
bnn_status run_im2col(const float *x, int N, int C, int H, int W, int kH, int kW, int sH, int sW, int pH, int pW,
                      uint64_t *cols, void *workspace, hipStream_t s);

// 3x3 convolution of a 3-channel image with fp32 NCHW output (conv.hip); validated arguments.
bnn_status launch_conv2d_f32_k27(const float *x, const float *w, int N, int H, int W, int D, int sH, int sW, int pH,
                                 int pW, const float *scale, const float *bias, float *out, hipStream_t s);

}  // namespace bnn
