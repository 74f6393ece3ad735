// Locality reordering of a row block's graph: symmetric permutation of a square CSR matrix by
// partition labels (Sec. 5 and Sec. 6.1: the vertices are renumbered so that every part owns a
// contiguous block of rows; A is permuted symmetrically and the rows of H follow).
//
//   perm / inv from labels   stable sort of the vertices by label (the order inside a part is
//                            the original order), done with the library's stable radix sort:
//                            the labels are the "column ids" of an n x n_parts pattern with one
//                            entry per row, whose transpose lists the vertices of every part
//   B = P A P^T              B[inv[r], inv[c]] = A[r, c].  Two stable transposes with a
//                            relabelling before each: relabel columns, transpose (rows are now
//                            new column ids, ascending, entries by old row), relabel those old
//                            row ids, transpose again (rows are new row ids, entries ascending
//                            by new column id, repeated entries in stored order).  Unique result.
// The dense side is moved with spmm_pack_rows: H_new = H[perm, :], Z_old = Z_new[inv, :].
// Integer work only: bit-exact.
#include "common.h"

namespace sagnn {
namespace {

constexpr int kThreads = 256;

inline dim3 grid_for(int64_t items) {
  int64_t b = ceil_div(items > 0 ? items : 1, kThreads);
  if (b > 256 * 32) b = 256 * 32;
  return dim3((unsigned)b);
}

__global__ __launch_bounds__(kThreads) void iota_kernel(int32_t* __restrict__ a, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) a[i] = (int32_t)i;
}

// out[i] = map[in[i]]; an id outside [0, n) sets err[0] and maps to 0
__global__ __launch_bounds__(kThreads) void relabel_kernel(const int32_t* __restrict__ in, int64_t cnt,
                                                           const int32_t* __restrict__ map, int64_t n,
                                                           int32_t* __restrict__ out,
                                                           int32_t* __restrict__ err) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < cnt; i += stride) {
    const int32_t c = in[i];
    if (c < 0 || c >= n) {
      err[0] = 1;
      out[i] = 0;
    } else {
      out[i] = map[c];
    }
  }
}

// inv[perm[i]] = i
__global__ __launch_bounds__(kThreads) void invert_kernel(const int32_t* __restrict__ perm, int64_t n,
                                                          int32_t* __restrict__ inv) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
    const int32_t p = perm[i];
    if (p >= 0 && p < n) inv[p] = (int32_t)i;
  }
}

// err[1] = 1 unless map is a permutation of [0, n): every value in range and seen exactly once
__global__ __launch_bounds__(kThreads) void check_perm_kernel(const int32_t* __restrict__ map, int64_t n,
                                                              int32_t* __restrict__ seen,
                                                              int32_t* __restrict__ err) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
    const int32_t p = map[i];
    if (p < 0 || p >= n) err[1] = 1;
    else if (atomicAdd(&seen[p], 1) != 0) err[1] = 1;
  }
}

__global__ __launch_bounds__(kThreads) void zero_i32_kernel(int32_t* __restrict__ a, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) a[i] = 0;
}

struct PermuteWs {
  int32_t *ci_a, *rp_b, *ci_b, *seen, *err;
  float* va_b;
  char* tws;
  size_t tws_bytes, bytes;
};

int carve_permute(void* base, int64_t n, int64_t nnz, PermuteWs* w) {
  size_t tb = 0;
  int rc = spmm_transpose_workspace_bytes(nnz, &tb);
  if (rc != SAGNN_OK) return rc;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char* p = base ? static_cast<char*>(base) + off : nullptr;
    off += round_up(bytes > 0 ? bytes : 4, 256);
    return p;
  };
  const size_t e = (size_t)(nnz > 0 ? nnz : 1);
  w->ci_a = reinterpret_cast<int32_t*>(take(4 * e));
  w->rp_b = reinterpret_cast<int32_t*>(take(4 * (size_t)(n + 1)));
  w->ci_b = reinterpret_cast<int32_t*>(take(4 * e));
  w->va_b = reinterpret_cast<float*>(take(4 * e));
  w->seen = reinterpret_cast<int32_t*>(take(4 * (size_t)(n > 0 ? n : 1)));
  w->err = reinterpret_cast<int32_t*>(take(16));
  w->tws = take(tb);
  w->tws_bytes = tb;
  w->bytes = off;
  return SAGNN_OK;
}

}  // namespace
}  // namespace sagnn

SAGNN_EXPORT int spmm_permute_workspace_bytes(int64_t n, int64_t nnz, size_t* bytes) {
  using namespace sagnn;
  if (!bytes || n < 0 || nnz < 0 || n > 0x7FFFFFFFll || nnz > 0x7FFFFFFFll) return SAGNN_EINVAL;
  PermuteWs w{};
  // the label sort transposes an n-entry pattern, the matrix permutation an nnz-entry one
  int rc = carve_permute(nullptr, n, nnz > n ? nnz : n, &w);
  if (rc != SAGNN_OK) return rc;
  *bytes = w.bytes;
  return SAGNN_OK;
}

SAGNN_EXPORT int spmm_perm_from_labels(const int32_t* d_labels, int64_t n, int32_t n_parts,
                                       int32_t* d_perm, int32_t* d_inv, int64_t* h_part_off,
                                       void* d_ws, size_t ws_bytes, void* stream) {
  using namespace sagnn;
  if (n < 0 || n > 0x7FFFFFFFll || n_parts < 1) return SAGNN_EINVAL;
  if (!d_perm || !d_inv || !h_part_off || !d_ws || (n > 0 && !d_labels)) return SAGNN_EINVAL;
  if (reinterpret_cast<uintptr_t>(d_ws) & 255u) return SAGNN_EINVAL;
  PermuteWs w{};
  int rc = carve_permute(d_ws, n, n, &w);
  if (rc != SAGNN_OK) return rc;
  if (ws_bytes < w.bytes) return SAGNN_ECAPACITY;
  hipStream_t s = (hipStream_t)stream;
  if (n_parts > 1024 || (int64_t)n_parts > (n > 0 ? n : 1)) return SAGNN_EINVAL;
  for (int32_t q = 0; q <= n_parts; ++q) h_part_off[q] = 0;
  if (n == 0) return SAGNN_OK;
  // pattern with one entry per row: rowptr = 0..n, column id = label, value unused
  hipLaunchKernelGGL(iota_kernel, grid_for(n + 1), dim3(kThreads), 0, s, w.ci_a, n + 1);
  SAGNN_LAUNCH_CHECK();
  // transpose: row q of the result lists the vertices with label q, ascending = the new order
  rc = spmm_csr_transpose(w.ci_a, d_labels, reinterpret_cast<const float*>(d_labels), n, n_parts, n,
                          w.rp_b, d_perm, w.va_b, w.tws, w.tws_bytes, stream);
  if (rc != SAGNN_OK) return rc;   // SAGNN_EFORMAT: a label outside [0, n_parts)
  hipLaunchKernelGGL(invert_kernel, grid_for(n), dim3(kThreads), 0, s, d_perm, n, d_inv);
  SAGNN_LAUNCH_CHECK();
  // part offsets -> host (32-bit on the device, widened here)
  int32_t stack_off[1025];
  SAGNN_HIP(hipMemcpyAsync(stack_off, w.rp_b, sizeof(int32_t) * (size_t)(n_parts + 1),
                           hipMemcpyDeviceToHost, s));
  SAGNN_HIP(hipStreamSynchronize(s));
  for (int32_t q = 0; q <= n_parts; ++q) h_part_off[q] = stack_off[q];
  return SAGNN_OK;
}

SAGNN_EXPORT int spmm_csr_permute_symmetric(const int32_t* d_rowptr, const int32_t* d_colidx,
                                            const float* d_val, int64_t n, int64_t nnz,
                                            const int32_t* d_inv, int32_t* d_rowptr_p,
                                            int32_t* d_colidx_p, float* d_val_p, void* d_ws,
                                            size_t ws_bytes, void* stream) {
  using namespace sagnn;
  if (n < 0 || nnz < 0 || n > 0x7FFFFFFFll || nnz > 0x7FFFFFFFll) return SAGNN_EINVAL;
  if (!d_rowptr || !d_rowptr_p || !d_ws || (n > 0 && !d_inv)) return SAGNN_EINVAL;
  if (nnz > 0 && (!d_colidx || !d_val || !d_colidx_p || !d_val_p)) return SAGNN_EINVAL;
  if (reinterpret_cast<uintptr_t>(d_ws) & 255u) return SAGNN_EINVAL;
  PermuteWs w{};
  int rc = carve_permute(d_ws, n, nnz, &w);
  if (rc != SAGNN_OK) return rc;
  if (ws_bytes < w.bytes) return SAGNN_ECAPACITY;
  hipStream_t s = (hipStream_t)stream;
  hipLaunchKernelGGL(zero_i32_kernel, grid_for(n + 4), dim3(kThreads), 0, s, w.seen, n);
  SAGNN_LAUNCH_CHECK();
  hipLaunchKernelGGL(zero_i32_kernel, dim3(1), dim3(kThreads), 0, s, w.err, 4);
  SAGNN_LAUNCH_CHECK();
  if (n > 0) {
    hipLaunchKernelGGL(check_perm_kernel, grid_for(n), dim3(kThreads), 0, s, d_inv, n, w.seen, w.err);
    SAGNN_LAUNCH_CHECK();
  }
  int32_t h_err[4] = {0, 0, 0, 0};
  SAGNN_HIP(hipMemcpyAsync(h_err, w.err, sizeof(h_err), hipMemcpyDeviceToHost, s));
  SAGNN_HIP(hipStreamSynchronize(s));
  if (h_err[1]) return SAGNN_EFORMAT;          // d_inv is not a permutation of [0, n)
  if (nnz > 0) {
    hipLaunchKernelGGL(relabel_kernel, grid_for(nnz), dim3(kThreads), 0, s, d_colidx, nnz, d_inv, n,
                       w.ci_a, w.err);
    SAGNN_LAUNCH_CHECK();
  }
  rc = spmm_csr_transpose(d_rowptr, w.ci_a, d_val, n, n, nnz, w.rp_b, w.ci_b, w.va_b, w.tws,
                          w.tws_bytes, stream);
  if (rc != SAGNN_OK) return rc;
  if (nnz > 0) {
    // ci_b holds old row ids (always in range); relabel them in place into ci_a
    hipLaunchKernelGGL(relabel_kernel, grid_for(nnz), dim3(kThreads), 0, s, w.ci_b, nnz, d_inv, n,
                       w.ci_a, w.err);
    SAGNN_LAUNCH_CHECK();
  }
  rc = spmm_csr_transpose(w.rp_b, w.ci_a, w.va_b, n, n, nnz, d_rowptr_p, d_colidx_p, d_val_p, w.tws,
                          w.tws_bytes, stream);
  if (rc != SAGNN_OK) return rc;
  SAGNN_HIP(hipMemcpyAsync(h_err, w.err, sizeof(h_err), hipMemcpyDeviceToHost, s));
  SAGNN_HIP(hipStreamSynchronize(s));
  if (h_err[0]) return SAGNN_EFORMAT;          // a column index outside [0, n)
  return SAGNN_OK;
}
