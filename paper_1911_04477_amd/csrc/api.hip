// Host-only parts of the C ABI: size helpers, status names, the kernel-timing hook.
#include <vector>

#include "common.h"
#include "bnn_testing.h"

extern "C" const char *bnn_status_str(bnn_status s) {
  switch (s) {
    case BNN_OK: return "BNN_OK";
    case BNN_ERR_NULL: return "BNN_ERR_NULL";
    case BNN_ERR_SHAPE: return "BNN_ERR_SHAPE";
    case BNN_ERR_STRIDE: return "BNN_ERR_STRIDE";
    case BNN_ERR_ALIGN: return "BNN_ERR_ALIGN";
    case BNN_ERR_WORKSPACE: return "BNN_ERR_WORKSPACE";
    case BNN_ERR_HIP: return "BNN_ERR_HIP";
    case BNN_ERR_UNSUPPORTED: return "BNN_ERR_UNSUPPORTED";
  }
  return "BNN_ERR_UNKNOWN";
}

extern "C" int64_t bnn_packed_words(int64_t K) { return K <= 0 ? 0 : (K + 63) / 64; }

extern "C" int64_t bnn_conv_kwords(int C, int kH, int kW) {
  if (C <= 0 || kH <= 0 || kW <= 0) return 0;
  return (int64_t)kH * kW * bnn_packed_words(C);
}

extern "C" int64_t bnn_conv_out_dim(int64_t in, int64_t k, int64_t stride, int64_t pad) {
  if (in <= 0 || k <= 0 || stride <= 0 || pad < 0) return 0;
  const int64_t span = in + 2 * pad - k;
  if (span < 0) return 0;
  return span / stride + 1;
}

// ---- kernel timing ---------------------------------------------------------------------
namespace bnn {
namespace {
struct ProfRecord {
  int kid;
  hipEvent_t e0, e1;
};
bool g_prof_on = false;
std::vector<ProfRecord> g_pool;  // events are created once and reused
int64_t g_used = 0;
bool g_open = false;
}  // namespace

void prof_begin(int kernel_id, hipStream_t s) {
  g_open = false;
  if (!g_prof_on || g_used >= BNN_PROF_MAX_RECORDS) return;
  if (g_used >= (int64_t)g_pool.size()) {
    ProfRecord r;
    r.kid = 0;
    if (hipEventCreate(&r.e0) != hipSuccess) return;
    if (hipEventCreate(&r.e1) != hipSuccess) {
      (void)hipEventDestroy(r.e0);
      return;
    }
    g_pool.push_back(r);
  }
  g_pool[g_used].kid = kernel_id;
  (void)hipEventRecord(g_pool[g_used].e0, s);
  g_open = true;
}

void prof_end(hipStream_t s) {
  if (!g_open) return;
  (void)hipEventRecord(g_pool[g_used].e1, s);
  ++g_used;
  g_open = false;
}
}  // namespace bnn

extern "C" bnn_status bnn_prof_enable(int enable) {
  using namespace bnn;
  g_prof_on = enable != 0;
  g_used = 0;
  if (!g_prof_on) {
    for (auto &r : g_pool) {
      (void)hipEventDestroy(r.e0);
      (void)hipEventDestroy(r.e1);
    }
    g_pool.clear();
  }
  return BNN_OK;
}

extern "C" bnn_status bnn_prof_reset(void) {
  bnn::g_used = 0;
  return BNN_OK;
}

extern "C" int64_t bnn_prof_count(void) { return bnn::g_used; }

extern "C" bnn_status bnn_prof_get(int64_t i, int *kernel_id, float *milliseconds) {
  using namespace bnn;
  if (!kernel_id || !milliseconds) return BNN_ERR_NULL;
  if (i < 0 || i >= g_used) return BNN_ERR_SHAPE;
  if (hipEventSynchronize(g_pool[i].e1) != hipSuccess) return BNN_ERR_HIP;
  float ms = 0.f;
  if (hipEventElapsedTime(&ms, g_pool[i].e0, g_pool[i].e1) != hipSuccess) return BNN_ERR_HIP;
  *kernel_id = g_pool[i].kid;
  *milliseconds = ms;
  return BNN_OK;
}

extern "C" const char *bnn_kernel_name(int kernel_id) {
  switch (kernel_id) {
    case bnn::KID_ENCODE_ROWS: return "encode_rows";
    case bnn::KID_PACK_CONV_WEIGHT: return "pack_conv_weight";
    case bnn::KID_ENCODE_NCHW: return "encode_nchw";
    case bnn::KID_IM2COL_GATHER: return "im2col_gather";
    case bnn::KID_XNOR_GEMM: return "xnor_gemm";
    case bnn::KID_XNOR_GEMM_SMALL: return "xnor_gemm_small";
    case bnn::KID_XNOR_GEMM_LOWK: return "xnor_gemm_lowk";
    case bnn::KID_XNOR_CONV_LATENCY: return "xnor_conv_latency";
    case bnn::KID_XNOR_GEMM_MFMA: return "xnor_gemm_mfma_i8";
    case bnn::KID_XNOR_GEMM_MFMA_FP4: return "xnor_gemm_mfma_fp4";
    case bnn::KID_XNOR_GEMM_MFMA_FP4X: return "xnor_gemm_mfma_fp4_expanded";
    case bnn::KID_EXPAND_FP4: return "expand_fp4";
    case bnn::KID_CONTROL_CONV_F32: return "control_conv_f32";
    case bnn::KID_MAXPOOL: return "maxpool2x2";
    case bnn::KID_CONV_F32: return "conv2d_f32";
    case bnn::KID_CONV_F32_SIGN: return "conv2d_f32_sign";
    case bnn::KID_FC_F32: return "fc_f32";
    case bnn::KID_VALU_PROBE: return "valu_probe";
    case bnn::KID_COPY_PROBE: return "copy_probe";
  }
  return "unknown";
}
