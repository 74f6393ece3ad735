// Device helpers shared by the SpMM kernels: per-lane vector types and the dense-row load.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sagnn {

template <int N> struct Vec { typedef float T __attribute__((ext_vector_type(N))); };
template <> struct Vec<1> { typedef float T; };

// buffer resource over `bytes` bytes starting at p (raw buffer, 32-bit data format)
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const float* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p), 0, (int)bytes, 0x00020000);
}

// One piece (FPL floats) of dense row `col` per lane; loff = lane's byte offset inside the row.
// BUF: hardware buffer load, the row's byte offset rides in a scalar register (one scalar
// multiply per entry, no vector address arithmetic, reads past the resource return 0); needs
// the addressed part of B to be smaller than 4 GiB.  Otherwise 64-bit global addressing.
template <int FPL, bool BUF>
__device__ __forceinline__ typename Vec<FPL>::T load_row(__amdgpu_buffer_rsrc_t rs, const float* B,
                                                         uint32_t col, uint32_t loff,
                                                         uint32_t row_bytes, int64_t ldb) {
  using vec = typename Vec<FPL>::T;
  if constexpr (BUF) {
    const uint32_t soff = col * row_bytes;
    if constexpr (FPL == 1) {
      return __builtin_bit_cast(vec, __builtin_amdgcn_raw_buffer_load_b32(rs, loff, soff, 0));
    } else if constexpr (FPL == 2) {
      return __builtin_bit_cast(vec, __builtin_amdgcn_raw_buffer_load_b64(rs, loff, soff, 0));
    } else {
      return __builtin_bit_cast(vec, __builtin_amdgcn_raw_buffer_load_b128(rs, loff, soff, 0));
    }
  } else {
    const char* rowbase = reinterpret_cast<const char*>(B + (int64_t)col * ldb);
    return *reinterpret_cast<const vec*>(rowbase + loff);
  }
}

// true if rows 0..kmax of width fw (leading dimension ldb) starting at B are addressable with a
// 32-bit byte offset; *bytes receives the size of that range
inline bool buffer_addressable(uint32_t kmax, int64_t ldb, int32_t fw, uint32_t* bytes) {
  const uint64_t reach = (uint64_t)kmax * (uint64_t)ldb * 4u + (uint64_t)fw * 4u;
  if (reach >= 0xFFFFFFFFull || (uint64_t)ldb * 4u >= 0xFFFFFFFFull) return false;
  *bytes = (uint32_t)reach;
  return true;
}

}  // namespace sagnn
