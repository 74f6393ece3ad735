// Internal helpers shared by the HIP translation units of libsagnn (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "sagnn.h"

#define SAGNN_EXPORT extern "C" __attribute__((visibility("default")))

namespace sagnn {

constexpr int kWave = 64;  // CDNA wavefront width

void set_hip_error(hipError_t e);

inline int hip_fail(hipError_t e) {
  set_hip_error(e);
  return SAGNN_EHIP;
}

#define SAGNN_HIP(expr)                                   \
  do {                                                    \
    hipError_t _e = (expr);                               \
    if (_e != hipSuccess) return ::sagnn::hip_fail(_e);   \
  } while (0)

// launch check: catches configuration errors without synchronising
#define SAGNN_LAUNCH_CHECK() SAGNN_HIP(hipGetLastError())

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// --- SpMM workspace geometry (host and device agree through these) -----------------------
// Entries per chunk of the nonzero-splitting schedule.  One wavefront owns one chunk.
constexpr int kSpmmChunk = 256;
constexpr uint32_t kSpmmMagic = 0x53A66E01u;

struct SpmmWsHeader {      // first 256 bytes of the SpMM workspace
  uint32_t magic;
  int32_t has_empty_rows;  // set by prepare if some row has no entries
  int64_t m, nnz, nchunks;
  int32_t f;
};

// layout: header | chunk_row[nchunks+1] | rowend flags, 1 bit per entry | carry[nchunks*f]
inline int64_t spmm_nchunks(int64_t nnz) { return ceil_div(nnz, kSpmmChunk); }
inline size_t spmm_ws_table_off() { return 256; }
inline size_t spmm_ws_flags_off(int64_t nnz) {
  return round_up(256 + sizeof(int32_t) * (size_t)(spmm_nchunks(nnz) + 1), 256);
}
inline size_t spmm_ws_carry_off(int64_t nnz) {  // flags padded to whole chunks
  return spmm_ws_flags_off(nnz) + round_up((size_t)spmm_nchunks(nnz) * (kSpmmChunk / 8), 256);
}
inline size_t spmm_ws_bytes(int64_t nnz, int32_t f) {
  return spmm_ws_carry_off(nnz) +
         round_up(sizeof(float) * (size_t)spmm_nchunks(nnz) * (size_t)f, 256);
}

// --- entry points implemented per translation unit (called by the layer functions) --------
int launch_spmm(const int32_t* rowptr, const int32_t* colidx, const float* val, int64_t m,
                int64_t k, int64_t nnz, const float* B, int64_t ldb, int32_t f, float* C,
                int64_t ldc, int32_t accumulate, void* ws, size_t ws_bytes, hipStream_t s);

int launch_gemm(const float* X, int64_t ldx, const float* W, int64_t ldw, int32_t transW,
                int64_t m, int32_t kdim, int32_t nout, int32_t prec, int32_t act,
                const float* mask, int64_t ldmask, float* Z, int64_t ldz, float* A, int64_t lda,
                hipStream_t s);

int launch_gemm_tn(const float* X, int64_t ldx, const float* S, int64_t lds_, int64_t m,
                   int32_t fi, int32_t fo, int32_t prec, float* Y, void* yws, size_t yws_bytes,
                   hipStream_t s);
size_t gemm_tn_ws_bytes(int64_t m, int32_t fi, int32_t fo);

}  // namespace sagnn
