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
constexpr uint32_t kSpmmMagic = 0x53A66E02u;

// Slab-sweep schedule (long rows): a wavefront owns kSweepSlots row pieces.
constexpr int kSweepSlots = 16;
// longest run of entries summed into one register before it is folded into the piece's slot
constexpr int kSweepRunMax = 128;
constexpr int kSweepMaxSlabs = 384;
constexpr int kSweepColBits = 27;           // column id bits in an encoded entry
constexpr int kSweepMinLong = 16;           // smallest degree a "long" row can be given

struct SpmmWsHeader {       // first 256 bytes of the SpMM workspace (device copy)
  uint32_t magic;
  int32_t has_empty_rows;   // some row of the matrix has no entries
  int64_t m, nnz;
  int32_t f;
  int32_t mode;             // 0: nonzero splitting over the caller's CSR; 1: slab sweep
  uint64_t generation;      // matches the host descriptor of the same prepare call
  // chunk part (the caller's CSR in mode 0, the short-row CSR in mode 1)
  int64_t c_rows, c_nnz, c_nchunks;
  // sweep part
  int64_t n_waves, n_long_entries, n_multi_rows, n_multi_pieces;
  int32_t n_slabs, slab_width;
  int32_t groups;           // lane groups per wavefront in the sweep streams (1, 2 or 4)
};
static_assert(sizeof(SpmmWsHeader) <= 256, "header must fit its slot");

// Fixed layout (a function of m, k, nnz, f only; every array has its worst-case size):
struct SpmmWsLayout {
  size_t header, chunk_row, flags, rowptr_s, rowmap_s, code, vals, piece_info, piece_target,
      wave_base, multi_row, multi_first, partial, carry, total;
  int64_t max_chunks, max_pieces, max_waves, max_multi_rows, max_multi_pieces, stream_cap;
};

inline int64_t spmm_nchunks(int64_t nnz) { return ceil_div(nnz, kSpmmChunk); }

inline SpmmWsLayout spmm_ws_layout(int64_t m, int64_t nnz, int32_t f) {
  SpmmWsLayout L{};
  L.max_chunks = spmm_nchunks(nnz) + 1;
  // every long row has >= kSweepMinLong entries; splitting adds at most nnz/1024 pieces
  L.max_pieces = nnz / kSweepMinLong + nnz / 1024 + kSweepSlots;
  L.max_waves = ceil_div(L.max_pieces, kSweepSlots) + 1;
  L.max_multi_rows = nnz / 1024 + 1;
  L.max_multi_pieces = 2 * (nnz / 1024) + 2;
  // sweep streams + gap + short CSR entries + padding.  A wavefront's stream is padded to the
  // batch of 8 steps; with lane groups (up to 4 zipped streams per wavefront) also to the longest
  // of its group streams, which the planner keeps within a small piece of each other.
  L.stream_cap = nnz + nnz / 8 + 64 * L.max_waves + 4 * kSpmmChunk;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += round_up(bytes, 256); return o; };
  L.header = take(256);
  L.chunk_row = take(sizeof(int32_t) * (size_t)(L.max_chunks + 1));
  L.flags = take((size_t)L.max_chunks * (kSpmmChunk / 8));
  L.rowptr_s = take(sizeof(int32_t) * (size_t)(m + 1));
  L.rowmap_s = take(sizeof(int32_t) * (size_t)(m + 1));
  L.code = take(sizeof(uint32_t) * (size_t)L.stream_cap);
  L.vals = take(sizeof(float) * (size_t)L.stream_cap);
  L.piece_info = take(sizeof(int32_t) * 2 * (size_t)(L.max_waves * kSweepSlots));
  L.piece_target = take(sizeof(int32_t) * (size_t)(L.max_waves * kSweepSlots));
  L.wave_base = take(sizeof(int32_t) * (size_t)(L.max_waves + 1));
  L.multi_row = take(sizeof(int32_t) * (size_t)L.max_multi_rows);
  L.multi_first = take(sizeof(int32_t) * (size_t)(L.max_multi_rows + 1));
  L.partial = take(sizeof(float) * (size_t)L.max_multi_pieces * (size_t)f);
  L.carry = take(sizeof(float) * (size_t)L.max_chunks * (size_t)f);
  L.total = off;
  return L;
}
inline size_t spmm_ws_bytes(int64_t m, int64_t nnz, int32_t f) { return spmm_ws_layout(m, nnz, f).total; }

// Host descriptor of a prepared workspace (what the launcher needs without reading the device)
struct SpmmHostDesc {
  uint64_t generation;
  int64_t m, nnz;
  int32_t f, mode;
  int64_t c_rows, c_nnz, c_nchunks;
  int64_t n_waves, n_multi_rows, sweep_stream_len;
  int32_t has_empty_rows;
  int32_t groups;
  int64_t k;                // rows of B the schedule was prepared for (stream columns are < k)
};
void spmm_desc_put(const void* ws, const SpmmHostDesc& d);
bool spmm_desc_get(const void* ws, SpmmHostDesc* d);
void spmm_desc_erase(const void* ws);

// --- entry points implemented per translation unit (called by the layer functions) --------
int launch_spmm(const int32_t* rowptr, const int32_t* colidx, const float* val, int64_t m,
                int64_t k, int64_t nnz, const float* B, int64_t ldb, int32_t f, float* C,
                int64_t ldc, int32_t accumulate, void* ws, size_t ws_bytes, hipStream_t s);

// slab-sweep part (spmm_sweep.hip)
struct SweepPlanResult {
  bool use_sweep;
  SpmmWsHeader hdr;  // filled in for mode 1 (sweep part + short CSR sizes)
};
int sweep_prepare(const int32_t* d_rowptr, const int32_t* d_colidx, const float* d_val, int64_t m,
                  int64_t k, int64_t nnz, int32_t f, char* ws, const SpmmWsLayout& L,
                  hipStream_t s, SweepPlanResult* out);
// Planner parameters a tuning call may set for the next sweep_prepare() of this thread
// (0 = the default; environment overrides win over both).
struct SweepTuning {
  int piece;      // longest piece a long row is cut into
  int min_long;   // long-row threshold used where the planner would pick 64
};
void sweep_set_tuning(SweepTuning t);
int sweep_launch(const SpmmHostDesc& d, const SpmmWsLayout& L, char* ws, const float* B,
                 int64_t ldb, int32_t col0, int32_t fw, uint32_t kmax, float* C, int64_t ldc,
                 int32_t accumulate, int32_t f_total, hipStream_t s);

int launch_gemm(const float* X, int64_t ldx, const float* W, int64_t ldw, int32_t transW,
                int64_t m, int32_t kdim, int32_t nout, int32_t prec, int32_t act,
                const float* mask, int64_t ldmask, float* Z, int64_t ldz, float* A, int64_t lda,
                hipStream_t s);

int launch_gemm_tn(const float* X, int64_t ldx, const float* S, int64_t lds_, int64_t m,
                   int32_t fi, int32_t fo, int32_t prec, float* Y, void* yws, size_t yws_bytes,
                   hipStream_t s);
size_t gemm_tn_ws_bytes(int64_t m, int32_t fi, int32_t fo);

}  // namespace sagnn
