// Row pack / gather: out[r,:] = H[rows[r],:]  (Alg. 1, first statement: the packed buffer T
// is the concatenation of the needed rows of H; Alg. 2 "H[srows,:]").
//
// Pure HBM traffic: N*f*4 bytes read, N*f*4 written, N*4 bytes of indices.  Each lane moves
// one 16-byte piece of a row, so a row of f floats is read by f/4 adjacent lanes (512
// contiguous bytes for f = 128) and written fully coalesced.  Every thread issues
// kUnroll independent loads before its first store to keep enough bytes in flight.
#include "common.h"

namespace sagnn {
namespace {

constexpr int kPackThreads = 256;
constexpr int kUnroll = 4;
typedef float vec4 __attribute__((ext_vector_type(4)));  // one 16-byte piece

// f4 = f/4 16-byte pieces per row.  blockDim = (px, py) with px a power of two <= 64 and
// px*py = kPackThreads, so a wavefront covers 64/px rows and px adjacent pieces of each; no
// integer division is needed.  A block owns kUnroll*py consecutive output rows.
__global__ __launch_bounds__(kPackThreads) void pack_rows_kernel(
    const vec4* __restrict__ H, int64_t n, int64_t ldh4, int32_t f4,
    const int32_t* __restrict__ rows, int64_t N, vec4* __restrict__ out, int64_t ldo4) {
  const int px = blockDim.x, py = blockDim.y;
  const int64_t r0 = (int64_t)blockIdx.x * (kUnroll * py) + threadIdx.y;
  int64_t src[kUnroll];
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const int64_t r = r0 + (int64_t)u * py;
    src[u] = -1;
    if (r < N) {
      const int64_t s = (int64_t)rows[r];
      if (s >= 0 && s < n) src[u] = s;
    }
  }
  for (int p = threadIdx.x; p < f4; p += px) {
    vec4 v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      v[u] = vec4(0.f);
      if (src[u] >= 0) v[u] = __builtin_nontemporal_load(&H[src[u] * ldh4 + p]);
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int64_t r = r0 + (int64_t)u * py;
      if (r < N) out[r * ldo4 + p] = v[u];
    }
  }
}

}  // namespace
}  // namespace sagnn

SAGNN_EXPORT int spmm_pack_rows(const float* d_H, int64_t n, int64_t ldh, int32_t f,
                                const int32_t* d_rows, int64_t N, float* d_out, int64_t ldo,
                                void* stream) {
  using namespace sagnn;
  if (n < 0 || N < 0 || f <= 0 || (f & 3) || ldh < f || ldo < f || (ldh & 3) || (ldo & 3))
    return SAGNN_EINVAL;
  if (N == 0) return SAGNN_OK;
  if (!d_H || !d_rows || !d_out || !aligned16(d_H) || !aligned16(d_out)) return SAGNN_EINVAL;
  const int32_t f4 = f / 4;
  int px = 1;
  while (px < f4 && px < 64) px <<= 1;
  const int py = kPackThreads / px;
  const int64_t blocks = ceil_div(N, (int64_t)kUnroll * py);
  if (blocks > 0x7FFFFFFFll) return SAGNN_EINVAL;
  hipLaunchKernelGGL(pack_rows_kernel, dim3((unsigned)blocks), dim3(px, py), 0,
                     (hipStream_t)stream, reinterpret_cast<const vec4*>(d_H), n, ldh / 4, f4,
                     d_rows, N, reinterpret_cast<vec4*>(d_out), ldo / 4);
  SAGNN_LAUNCH_CHECK();
  return SAGNN_OK;
}
