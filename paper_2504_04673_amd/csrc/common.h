// Internal helpers shared by the HIP translation units of libsagnn (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

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
// The sweep is cut into intervals of `sync_slabs` slabs; between two intervals the workgroups of
// an XCD that run at the same time wait for each other (bounded), so that they stay in the same
// part of B.  A wavefront's stream is padded to a whole batch at every interval boundary.
constexpr int kSweepMaxIntervals = 64;
constexpr int kSweepBarrierSlots = 65536;   // arrival counters (cohort x XCD x interval)
constexpr int kSweepMaxWindows = 2048;      // dealing windows of a matrix (11 bits of a sort key)

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
  int32_t n_intervals;      // >= 1; interval boundaries are barrier points when sync_slabs > 0
  int32_t sync_slabs;       // slabs per interval (0: no barriers, one interval)
  int32_t wg_per_cohort;    // workgroups that are resident together (a multiple of 8)
  int32_t sync_timeout_ticks;  // bounded wait at a barrier, in 100 MHz ticks
  int32_t sync_test_extra;  // test hook: added to the expected arrivals (forces the give-up path)
  int32_t slots;            // accumulator rows (pieces) per wavefront actually used, <= kSweepSlots
  int32_t barriers;         // 1: barriers at interval boundaries
  int32_t pace_ps_per_step; // pacing asked for at prepare time (0: none)
  int32_t max_slab;         // widest column slab of B per launch (256 or 128)
};
static_assert(sizeof(SpmmWsHeader) <= 256, "header must fit its slot");

// Fixed layout (a function of m, k, nnz, f only; every array has its worst-case size):
struct SpmmWsLayout {
  size_t header, chunk_row, flags, rowptr_s, rowmap_s, code, vals, piece_info, piece_target,
      wave_base, wave_steps, sync_off, barrier, sched, multi_row, multi_first, partial, carry, plan, wpack, total;
  int64_t max_chunks, max_pieces, max_waves, max_multi_rows, max_multi_pieces, stream_cap;
};

inline int64_t spmm_nchunks(int64_t nnz) { return ceil_div(nnz, kSpmmChunk); }

inline SpmmWsLayout spmm_ws_layout(int64_t m, int64_t nnz, int32_t f) {
  SpmmWsLayout L{};
  L.max_chunks = spmm_nchunks(nnz) + 1;
  // every long row has >= kSweepMinLong entries; splitting adds at most nnz/1024 pieces; every
  // short row may become a piece of its own (whole-row wavefronts behind those of the long rows)
  const int64_t long_pieces = nnz / kSweepMinLong + nnz / 1024 + kSweepSlots;
  const int64_t long_waves = ceil_div(long_pieces, kSweepSlots) + 1;
  const int64_t short_waves = ceil_div(m, kSweepSlots) + 4;
  L.max_pieces = long_pieces + m;
  L.max_waves = long_waves + short_waves;
  L.max_multi_rows = nnz / 1024 + 1;
  L.max_multi_pieces = 2 * (nnz / 1024) + 2;
  // sweep streams + gap + short CSR entries + padding.  A wavefront's stream is padded to the
  // batch of 8 steps at every interval boundary; with lane groups (up to 4 zipped streams per
  // wavefront) also to the longest of its group streams inside every interval.  If a pattern
  // needs more than this, the planner lays the streams out as one interval.  A whole-row
  // wavefront has one interval: at most 8 steps of padding for each of its up to 4 group streams.
  L.stream_cap = nnz + nnz / 4 + 256 * long_waves + 32 * short_waves + 4 * kSpmmChunk;
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
  L.wave_steps = take(sizeof(int32_t) * (size_t)(L.max_waves + 1));
  L.sync_off = take(sizeof(int32_t) * (size_t)L.max_waves * (kSweepMaxIntervals + 1));
  L.barrier = take(sizeof(uint32_t) * (size_t)(kSweepBarrierSlots + 64));
  L.sched = take(sizeof(float) * (size_t)(kSweepMaxIntervals + 2));
  L.multi_row = take(sizeof(int32_t) * (size_t)L.max_multi_rows);
  L.multi_first = take(sizeof(int32_t) * (size_t)(L.max_multi_rows + 1));
  L.partial = take(sizeof(float) * (size_t)L.max_multi_pieces * (size_t)f);
  L.carry = take(sizeof(float) * (size_t)L.max_chunks * (size_t)f);
  // planner: totals, per-window arrays, tile sums of the five row scans (2048 rows per tile)
  L.plan = take(256 + (size_t)kSweepMaxWindows * 8 + 3 * 4 * (size_t)(kSweepMaxWindows + 64) +
                5 * sizeof(int32_t) * (size_t)(ceil_div(m, 2048) + 2));
  // W of a fused layer call packed for the bfloat16 matrix instructions (at most 256 x 256, up to
  // three terms per element)
  L.wpack = take(3 * 256 * 256 * 2);
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
  int32_t n_intervals, sync_slabs, wg_per_cohort, sync_timeout_ticks, sync_test_extra;
  int32_t slots;
  int32_t barriers, pace_ps_per_step;
  int32_t max_slab;         // widest column slab of B per launch (256, or 128 for the lane-group kernels at wider f)
  float mean_steps;         // average stream steps per wavefront (the end of the pacing schedule)
  float max_steps;          // steps of the longest stream
  // dense-tile schedule (tiles.hip): when tiles != 0 everything above describes the rest CSR
  // stored in the tile region behind the plain workspace, nnz included; full_nnz is the caller's
  int32_t tiles;
  int64_t full_nnz, tile_count, tile_items, tile_entries, tile_rows;
  uint64_t tile_generation;
};

// Workgroups of `lds` bytes of LDS each that a CU really holds at once.  Measured on MI355X:
// 5 x 32000 bytes fit, 5 x 32768 do not (the runtime's occupancy query says 5 for both), 2 x 65536
// fit, 3 x 53248 were not tried.  Modelled as 160 KB minus 2 KB, allocations rounded up to 1280
// bytes; an estimate on the low side is harmless wherever this is used.
inline int lds_resident_workgroups(size_t lds) {
  const size_t unit = round_up(lds > 0 ? lds : 1, 1280);
  size_t n = (160u * 1024u - 2048u) / unit;
  if (n > 8) n = 8;   // 32 wavefronts per CU, four per workgroup
  return (int)n;
}
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
  float mean_steps;  // average stream steps per wavefront
  float max_steps;   // steps of the longest stream
  SpmmWsHeader hdr;  // filled in for mode 1 (sweep part + short CSR sizes)
};
int sweep_prepare(const int32_t* d_rowptr, const int32_t* d_colidx, const float* d_val, int64_t m,
                  int64_t k, int64_t nnz, int32_t f, char* ws, const SpmmWsLayout& L,
                  const sagnn_spmm_options& opt, hipStream_t s, SweepPlanResult* out);
// device side of the planner (sweep_plan.hip); the scratch arrays live in the stream arrays of the
// workspace, which are written last
struct SweepRowTotals {
  int64_t pieces, short_rows, short_entries, multi_rows, multi_pieces;
  int32_t min_long;
  bool has_empty, bad;
};
bool sweep_plan_fits(const SpmmWsLayout& L);
// classify rows, build the short-row CSR, the list of split rows and the piece records; one
// stream synchronisation (a 128-byte copy)
// (short_pieces: the short rows also get piece records, one whole row each, behind those of the long rows)
int sweep_plan_rows(const int32_t* d_rowptr, int64_t m, int64_t nnz, int32_t opt_min_long, int32_t piece_max,
                    char* ws, const SpmmWsLayout& L, hipStream_t s, SweepRowTotals* out, bool short_pieces = false);
// entries of the pieces of every window (only needed with several windows; synchronises)
int sweep_plan_window_entries(char* ws, const SpmmWsLayout& L, int64_t P, int64_t window, int32_t nwin,
                              hipStream_t s, std::vector<int64_t>* entries);
// sort the pieces and deal them to the streams: fills piece_info / piece_target; synchronises
// (it looks at a flag every few batches to see whether pieces are left); flags[2] of the carry
// area stays 1 if pieces were left over
int sweep_plan_deal(char* ws, const SpmmWsLayout& L, int64_t P, int64_t window, const int32_t* h_win_unit0,
                    int32_t nwin, int64_t n_waves4, int32_t R, int32_t SL, bool snake, hipStream_t s);
// the short rows' pieces (records P_long .. P_long + n_short), longest first, 16 consecutive ones
// per wavefront from wavefront first_wave on (n_waves4 of sweep_plan_deal must cover them); no
// synchronisation
int sweep_plan_deal_short(char* ws, const SpmmWsLayout& L, int64_t P_long, int64_t n_short, int64_t first_wave,
                          hipStream_t s);
// the sweep with the dense transform of a GCN layer as its epilogue (spmm_sweep.hip)
struct SweepFusedArgs {
  const float* W;        // f_in x f_out, row-major
  const void* Wp;        // bfloat16 products: W packed for the matrix cores (set by the launcher)
  float *Z, *Hout, *T;   // m x f_out, m x f_out, m x f_in; each may be NULL (not both Z and Hout)
  int32_t f_out, act;
};
int sweep_launch_fused(const SpmmHostDesc& d, const SpmmWsLayout& L, char* ws, const float* B, int64_t ldb,
                       int32_t f_in, uint32_t kmax, const SweepFusedArgs& fa, int32_t mode, hipStream_t s);
// the layer through that kernel plus a small kernel for the rows it leaves out (spmm.hip);
// returns 1 if the workspace / shapes do not allow it (the caller then uses another form)
bool fused_sweep_layer_applicable(const void* ws, int32_t f_in, int32_t f_out);
int launch_fused_sweep_layer(const int32_t* rowptr, const int32_t* colidx, const float* val, int64_t m,
                             int64_t k, int64_t nnz, const float* H, int64_t ldh, int32_t f_in,
                             const float* W, int32_t f_out, int32_t act, int32_t prec, float* T, float* Z,
                             float* Hout, void* ws, size_t ws_bytes, hipStream_t s);
// `fused` / `fuse` (lane-group schedules only): the layer form, see SweepFusedArgs
int sweep_launch(const SpmmHostDesc& d, const SpmmWsLayout& L, char* ws, const float* B,
                 int64_t ldb, int32_t col0, int32_t fw, uint32_t kmax, float* C, int64_t ldc,
                 int32_t accumulate, int32_t f_total, hipStream_t s,
                 const SweepFusedArgs* fused = nullptr, int32_t fuse = 0);

// Dense-tile schedule (tiles.hip): the tiles of A that are dense enough to re-use staged rows of
// the dense operand are multiplied out of LDS, the rest of A goes through the other schedules.
constexpr int64_t kTileMaxRows = 131072;   // ranked rows / columns that can form tiles
constexpr int64_t kTileMaxCols = 65536;
constexpr int64_t kTileItemEntries = 32768;   // entries of a work item (several tiles of one row group)
struct TileGeom { int fpl, rpw, rg, tc; };    // floats per lane, rows per wavefront, rows per group, columns per tile
bool tile_geom(int32_t f, TileGeom* g);       // false: no tile kernel for this width
struct TileWsLayout {   // the tile region (a function of m, k, nnz, f; worst-case sizes)
  size_t header, rowrank, colrank, hubrow, hubcol, tilecnt, tileslot, ts_chunk, ts_item, item_g, item_ts0,
      item_nch, group_item0, cnt16, roff16, wstart, ent, partial, rest_rowptr, rest_col, rest_val, keys, colcnt,
      err, radix, total;
  int64_t kr, kc, ng, nc, max_ts, max_items;
};
TileWsLayout tile_ws_layout(int64_t m, int64_t k, int64_t nnz, int32_t f);
struct TilePlan { int64_t n_ts, n_items, entries, rest_nnz, rows; };
int tile_prepare(const int32_t* d_rowptr, const int32_t* d_colidx, const float* d_val, int64_t m, int64_t k,
                 int64_t nnz, int32_t f, char* base, const TileWsLayout& L, int32_t reuse_x10, uint64_t generation,
                 hipStream_t s, TilePlan* out);
// C += (kept tiles of A) * B
int tile_launch(const TilePlan& p, uint64_t generation, char* base, const TileWsLayout& L, const float* B,
                int64_t ldb, uint32_t kmax, int32_t f, int64_t m, float* C, int64_t ldc, hipStream_t s);

// Stable least-significant-digit radix sort of (key, payload) pairs on the device (stages.hip),
// 8 bits per pass over key bits [0, bits).  With pay_in == NULL the payload is the index of the
// pair.  The sorted pairs end up in w.keys[*result], w.pay[*result].  A workspace carved for n
// pairs serves any smaller count.
struct RadixWs {
  uint32_t *keys[2], *pay[2];
  int32_t* counts;     // [256][ntiles + 1]
  int32_t* tilesum;    // [256][nscan + 1]
  int64_t* digit_off;  // [257]
  int64_t ntiles, nscan;
  int64_t cap;         // pairs the workspace was carved for
  size_t bytes;
};
RadixWs carve_radix(void* base, int64_t n);   // base == NULL: sizes only
int radix_sort_pairs(const uint32_t* keys_in, const uint32_t* pay_in, int64_t n, int bits, const RadixWs& w,
                     hipStream_t s, int* result);

int launch_gemm(const float* X, int64_t ldx, const float* W, int64_t ldw, int32_t transW,
                int64_t m, int32_t kdim, int32_t nout, int32_t prec, int32_t act,
                const float* mask, int64_t ldmask, float* Z, int64_t ldz, float* A, int64_t lda,
                hipStream_t s);

// fused layer forward (fused.hip): T = A H stays on the chip; T may be NULL
bool fused_layer_supported(int32_t f_in, int32_t f_out, int32_t prec);
int launch_fused_layer(const int32_t* rowptr, const int32_t* colidx, const float* val, int64_t m,
                       int64_t k, int64_t nnz, const float* H, int64_t ldh, int32_t f_in,
                       const float* W, int32_t f_out, int32_t act, int32_t prec, float* T, float* Z,
                       float* Hout, hipStream_t s);

int launch_gemm_tn(const float* X, int64_t ldx, const float* S, int64_t lds_, int64_t m,
                   int32_t fi, int32_t fo, int32_t prec, float* Y, void* yws, size_t yws_bytes,
                   hipStream_t s);
size_t gemm_tn_ws_bytes(int64_t m, int32_t fi, int32_t fo);

}  // namespace sagnn
