// C-ABI glue: error reporting and the layer-level entry points that chain the kernels of
// spmm.hip and gemm.hip on one stream (Sec. 2.1 forward / backward equations, in the order
// of Alg. 1: sparse product first, dense transform second).
#include <atomic>
#include <mutex>
#include <unordered_map>

#include "common.h"

namespace sagnn {
namespace {
std::atomic<int> g_last_hip_error{0};
// host descriptors of prepared SpMM workspaces, keyed by the workspace address
std::mutex g_desc_mutex;
std::unordered_map<const void*, SpmmHostDesc> g_desc;
}  // namespace
void set_hip_error(hipError_t e) { g_last_hip_error.store((int)e); }
void spmm_desc_put(const void* ws, const SpmmHostDesc& d) {
  std::lock_guard<std::mutex> lock(g_desc_mutex);
  g_desc[ws] = d;
}
void spmm_desc_erase(const void* ws) {
  std::lock_guard<std::mutex> lock(g_desc_mutex);
  g_desc.erase(ws);
}
bool spmm_desc_get(const void* ws, SpmmHostDesc* d) {
  std::lock_guard<std::mutex> lock(g_desc_mutex);
  auto it = g_desc.find(ws);
  if (it == g_desc.end()) return false;
  *d = it->second;
  return true;
}
}  // namespace sagnn

SAGNN_EXPORT const char* sagnn_strerror(int code) {
  switch (code) {
    case SAGNN_OK: return "ok";
    case SAGNN_EINVAL: return "invalid argument (null, negative, misaligned or unsupported size)";
    case SAGNN_ECAPACITY: return "output buffer or workspace too small";
    case SAGNN_EFORMAT: return "malformed CSR or block offsets";
    case SAGNN_EHIP: return "HIP runtime call failed";
    default: return "unknown error";
  }
}

SAGNN_EXPORT int sagnn_last_hip_error(void) { return sagnn::g_last_hip_error.load(); }

SAGNN_EXPORT int sagnn_version(void) { return 200; }

SAGNN_EXPORT int spmm_csr_release(const void* d_ws) {
  if (!d_ws) return SAGNN_EINVAL;
  sagnn::spmm_desc_erase(d_ws);
  return SAGNN_OK;
}

SAGNN_EXPORT int gcn_layer_fwd(const int32_t* d_rowptr, const int32_t* d_colidx,
                               const float* d_val, int64_t m, int64_t k, int64_t nnz,
                               const float* d_H, int64_t ldh, int32_t f_in, const float* d_W,
                               int32_t f_out, int32_t act, int32_t gemm_prec, float* d_T,
                               float* d_Z, float* d_Hout, void* d_ws, size_t ws_bytes,
                               void* stream) {
  using namespace sagnn;
  if ((!d_Z && !d_Hout) || !d_W) return SAGNN_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  if (!d_T) {   // the caller does not want T: the rows of T never leave the chip
    if (d_ws) {
      // a workspace prepared for the one-row-per-instruction sweep whose wavefronts finish (nearly)
      // all rows: the sweep itself ends with the dense transform
      const int rc = launch_fused_sweep_layer(d_rowptr, d_colidx, d_val, m, k, nnz, d_H, ldh, f_in, d_W, f_out,
                                              act, gemm_prec, nullptr, d_Z, d_Hout, d_ws, ws_bytes, s);
      if (rc != 1) return rc;
    }
    return launch_fused_layer(d_rowptr, d_colidx, d_val, m, k, nnz, d_H, ldh, f_in, d_W, f_out, act,
                              gemm_prec, nullptr, d_Z, d_Hout, s);
  }
  int rc = launch_spmm(d_rowptr, d_colidx, d_val, m, k, nnz, d_H, ldh, f_in, d_T, f_in, 0, d_ws,
                       ws_bytes, s);
  if (rc != SAGNN_OK) return rc;
  return launch_gemm(d_T, f_in, d_W, f_out, 0, m, f_in, f_out, gemm_prec, act, nullptr, 0, d_Z,
                     f_out, d_Hout, f_out, s);
}

SAGNN_EXPORT int gcn_layer_fwd_fused(const int32_t* d_rowptr, const int32_t* d_colidx,
                                     const float* d_val, int64_t m, int64_t k, int64_t nnz,
                                     const float* d_H, int64_t ldh, int32_t f_in, const float* d_W,
                                     int32_t f_out, int32_t act, int32_t gemm_prec, float* d_T,
                                     float* d_Z, float* d_Hout, void* stream) {
  return sagnn::launch_fused_layer(d_rowptr, d_colidx, d_val, m, k, nnz, d_H, ldh, f_in, d_W, f_out,
                                   act, gemm_prec, d_T, d_Z, d_Hout, (hipStream_t)stream);
}

SAGNN_EXPORT int gcn_layer_fwd_form(const void* d_ws, int32_t f_in, int32_t f_out, int32_t gemm_prec,
                                    int32_t* h_form) {
  using namespace sagnn;
  if (!h_form) return SAGNN_EINVAL;
  if (d_ws && fused_sweep_layer_applicable(d_ws, f_in, f_out)) *h_form = 2;
  else *h_form = fused_layer_supported(f_in, f_out, gemm_prec) ? 1 : 0;
  return SAGNN_OK;
}

SAGNN_EXPORT int gcn_bwd_workspace_bytes(int64_t m, int32_t f_in, int32_t f_out, size_t* bytes) {
  using namespace sagnn;
  if (!bytes || m < 0 || f_in <= 0 || f_out <= 0 || (f_in & 3) || (f_out & 3) || f_in > 256 ||
      f_out > 256)
    return SAGNN_EINVAL;
  *bytes = gemm_tn_ws_bytes(m, f_in, f_out);
  return SAGNN_OK;
}

SAGNN_EXPORT int gcn_layer_bwd(const int32_t* d_rowptr, const int32_t* d_colidx,
                               const float* d_val, int64_t m, int64_t nnz, const float* d_G,
                               int32_t f_out, const float* d_W, int32_t f_in,
                               const float* d_Zprev, const float* d_Hprev, int32_t gemm_prec,
                               float* d_S, float* d_Gprev, float* d_Y, void* d_ws, size_t ws_bytes,
                               void* d_yws, size_t yws_bytes, void* stream) {
  using namespace sagnn;
  if (!d_S || !d_G) return SAGNN_EINVAL;
  if (d_Gprev && !d_W) return SAGNN_EINVAL;
  if (d_Y && (!d_Hprev || !d_yws)) return SAGNN_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  // S = A G : the same sparse product as the forward pass, on the gradient matrix
  int rc = launch_spmm(d_rowptr, d_colidx, d_val, m, m, nnz, d_G, f_out, f_out, d_S, f_out, 0,
                       d_ws, ws_bytes, s);
  if (rc != SAGNN_OK) return rc;
  if (d_Gprev) {
    // Gprev = (S W^T) .* [Zprev > 0];  W is f_in x f_out, so W^T is the stored matrix read
    // with transW = 1 (kdim = f_out, nout = f_in)
    rc = launch_gemm(d_S, f_out, d_W, f_out, 1, m, f_out, f_in, gemm_prec, SAGNN_ACT_IDENTITY,
                     d_Zprev, f_in, d_Gprev, f_in, nullptr, 0, s);
    if (rc != SAGNN_OK) return rc;
  }
  if (d_Y) {
    rc = launch_gemm_tn(d_Hprev, f_in, d_S, f_out, m, f_in, f_out, gemm_prec, d_Y, d_yws,
                        yws_bytes, s);
    if (rc != SAGNN_OK) return rc;
  }
  return SAGNN_OK;
}
