// Device side of the slab-sweep planner (one-time preparation of the local SpMM of Alg. 1 / 2;
// the sparsity pattern is fixed for a training run, Sec. 4.1, so this runs once per matrix).
//
//   rows    one pass classifies the rows (empty / short / long, where "long" starts at a degree
//           chosen from the degree distribution), a three-kernel scan turns the per-row counts
//           into positions, and the same pass run again emits: the compacted row pointer and
//           row map of the short rows, the list of rows that are cut into several pieces, and
//           one record per piece (row, piece index and count, size, partial-row slot).
//   sort    pieces are ordered by (window, size descending) with a stable radix sort; inside a
//           size class the row order is kept.
//   deal    largest piece first, each to the stream that is shortest so far and still has a free
//           accumulator slot.  The sequential rule is applied in batches: the next B pieces
//           (B = half the window's streams) go, in order, to the B shortest streams with a free
//           slot, found by sorting the streams by length.  On power-law graphs the stream
//           lengths come out as with the piece-by-piece rule (the pieces of a batch have nearly
//           equal sizes; where the slots per stream bind, the longest stream is about 1 % longer);
//           whole rounds (B = all streams) do not: the first round hands out the large pieces and
//           the later, much smaller ones cannot level them.
// The host only sees five totals (one 128-byte copy) and, for matrices of several windows, the
// entries per window.
#include <algorithm>
#include <vector>

#include "common.h"

namespace sagnn {
namespace {

constexpr int kT = 256;
constexpr int kRowTile = kT * 8;          // rows per workgroup in the row passes
constexpr uint32_t kFullUnit = 0xFFFFFFFFu;

enum Stat : int {
  ST_MID = 0,       // entries in rows of kSweepMinLong..63 entries
  ST_EMPTY,         // rows without entries
  ST_BAD,           // != 0: not a CSR row pointer for this nnz, or a row needs too many pieces
  ST_MINLONG,       // the degree from which a row is swept
  ST_PIECES,        // five totals of the row scan, in the order of RowQ
  ST_SHORT_ROWS,
  ST_SHORT_ENTRIES,
  ST_MULTI_ROWS,
  ST_MULTI_PIECES,
  ST_COUNT = 16
};

__global__ __launch_bounds__(kT) void plan_zero_kernel(unsigned long long* __restrict__ stat, int32_t* __restrict__ flags) {
  if (threadIdx.x < ST_COUNT) stat[threadIdx.x] = 0ull;
  if (threadIdx.x < 4) flags[threadIdx.x] = 0;
}

__global__ __launch_bounds__(kT) void plan_rowstat_kernel(const int32_t* __restrict__ rowptr, int64_t m,
                                                          int64_t nnz, unsigned long long* __restrict__ stat) {
  long long mid = 0, empty = 0, bad = 0;
  const int64_t stride = (int64_t)gridDim.x * kT;
  for (int64_t r = (int64_t)blockIdx.x * kT + threadIdx.x; r < m; r += stride) {
    const int64_t d = (int64_t)rowptr[r + 1] - rowptr[r];
    if (d < 0) bad = 1;
    else if (d == 0) ++empty;
    else if (d >= kSweepMinLong && d < 64) mid += d;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0 && (rowptr[0] != 0 || (int64_t)rowptr[m] != nnz)) bad = 1;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    mid += __shfl_down(mid, o, 64);
    empty += __shfl_down(empty, o, 64);
    bad += __shfl_down(bad, o, 64);
  }
  if ((threadIdx.x & 63) == 0) {
    if (mid) atomicAdd(&stat[ST_MID], (unsigned long long)mid);
    if (empty) atomicAdd(&stat[ST_EMPTY], (unsigned long long)empty);
    if (bad) atomicAdd(&stat[ST_BAD], (unsigned long long)bad);
  }
}

// Rows with at least min_long entries go through the sweep.  64 suits power-law graphs (the many
// rows below it hold few entries and would only add accumulator slots); when the rows of 16..63
// entries hold a large share of the matrix (near-regular graphs, e.g. a partitioned graph's row
// block) the threshold drops so that they are swept too.  opt > 0: forced; opt < 0: -opt is used
// where the rule would pick 64.
__global__ void plan_rule_kernel(unsigned long long* __restrict__ stat, int64_t nnz, int32_t opt_min_long) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  int32_t min_long = opt_min_long;
  if (min_long <= 0)
    min_long = ((long long)stat[ST_MID] * 4 >= nnz) ? kSweepMinLong : (min_long < 0 ? -min_long : 64);
  if (min_long < kSweepMinLong) min_long = kSweepMinLong;
  stat[ST_MINLONG] = (unsigned long long)min_long;
}

struct RowQ {
  int v[5];   // pieces, short row (0/1), entries if short, cut into several pieces (0/1), pieces if so
};

__device__ __forceinline__ RowQ row_q(int64_t d, int32_t min_long, int32_t piece_max, bool* too_many) {
  RowQ q{};
  if (d >= min_long) {
    const int64_t p = (d + piece_max - 1) / piece_max;
    if (p > 0x7FFF) { *too_many = true; return q; }
    q.v[0] = (int)p;
    q.v[3] = p > 1;
    q.v[4] = p > 1 ? (int)p : 0;
  } else if (d > 0) {
    q.v[1] = 1;
    q.v[2] = (int)d;
  }
  return q;
}

// exclusive scan over the workgroup of five per-thread sums; tot[] = workgroup totals
__device__ __forceinline__ void block_scan5(const int (&s)[5], int (&ex)[5], int (&tot)[5]) {
  __shared__ int wsum[kT / 64][5];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc[5];
#pragma unroll
  for (int c = 0; c < 5; ++c) {
    int v = s[c];
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int t = __shfl_up(v, d, 64);
      if (lane >= d) v += t;
    }
    inc[c] = v;
    if (lane == 63) wsum[wave][c] = v;
  }
  __syncthreads();
#pragma unroll
  for (int c = 0; c < 5; ++c) {
    int base = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kT / 64; ++w) {
      if (w < wave) base += wsum[w][c];
      total += wsum[w][c];
    }
    ex[c] = base + inc[c] - s[c];
    tot[c] = total;
  }
  __syncthreads();
}

struct PieceArrays {
  int32_t *row, *jp, *size, *mf;   // jp = piece index << 16 | pieces of the row; mf = partial-row slot or -1
};

// EMIT = false: tilesum[c][tile] = sums of the tile's rows.  EMIT = true (tile sums scanned):
// write what the positions address.
template <bool EMIT>
__global__ __launch_bounds__(kT) void plan_rows_kernel(
    const int32_t* __restrict__ rowptr, int64_t m, int32_t piece_max, int64_t ntiles,
    unsigned long long* __restrict__ stat, int32_t* __restrict__ tilesum, int32_t* __restrict__ rowptr_s,
    int32_t* __restrict__ rowmap_s, int32_t* __restrict__ multi_row, int32_t* __restrict__ multi_first,
    PieceArrays pa, int64_t max_pieces, int64_t max_multi_rows, int32_t short_pieces) {
  const int32_t min_long = (int32_t)stat[ST_MINLONG];
  const int64_t r0 = (int64_t)blockIdx.x * kRowTile + (int64_t)threadIdx.x * 8;
  RowQ q[8];
  int64_t deg[8];
  int s[5] = {0, 0, 0, 0, 0};
  bool too_many = false;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int64_t r = r0 + i;
    deg[i] = r < m ? (int64_t)rowptr[r + 1] - rowptr[r] : 0;
    q[i] = row_q(deg[i], min_long, piece_max, &too_many);
#pragma unroll
    for (int c = 0; c < 5; ++c) s[c] += q[i].v[c];
  }
  int ex[5], tot[5];
  block_scan5(s, ex, tot);
  if (!EMIT) {
    if (too_many) atomicAdd(&stat[ST_BAD], 1ull);
    if (threadIdx.x == 0) {
#pragma unroll
      for (int c = 0; c < 5; ++c) tilesum[(int64_t)c * (ntiles + 1) + blockIdx.x] = tot[c];
    }
    return;
  }
  int64_t run[5];
#pragma unroll
  for (int c = 0; c < 5; ++c) run[c] = (int64_t)tilesum[(int64_t)c * (ntiles + 1) + blockIdx.x] + ex[c];
  // short_pieces: every short row also gets a piece record (one whole-row piece), stored behind
  // the pieces of the long rows in row order, for the schedules that sweep the short rows too
  const int64_t short_id0 = (int64_t)stat[ST_PIECES];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int64_t r = r0 + i;
    if (r < m) {
      if (q[i].v[1]) {
        rowptr_s[run[1]] = (int32_t)run[2];
        rowmap_s[run[1]] = (int32_t)r;
        const int64_t id = short_id0 + run[1];
        if (short_pieces && id < max_pieces) {
          pa.row[id] = (int32_t)r;
          pa.jp[id] = 1;                 // piece 0 of 1
          pa.size[id] = (int32_t)deg[i];
          pa.mf[id] = -1;
        }
      }
      const int p = q[i].v[0];
      if (q[i].v[3] && run[3] < max_multi_rows) {
        multi_row[run[3]] = (int32_t)r;
        multi_first[run[3]] = (int32_t)run[4];
      }
      for (int j = 0; j < p; ++j) {
        const int64_t id = run[0] + j;
        if (id < max_pieces) {
          pa.row[id] = (int32_t)r;
          pa.jp[id] = (j << 16) | p;
          pa.size[id] = (int32_t)((deg[i] - j + p - 1) / p);
          pa.mf[id] = p > 1 ? (int32_t)(run[4] + j) : -1;
        }
      }
    }
#pragma unroll
    for (int c = 0; c < 5; ++c) run[c] += q[i].v[c];
  }
}

// one workgroup: exclusive scan of the five rows of tile sums; totals to stat and to the ends of
// the two arrays that are indexed with a count
__global__ __launch_bounds__(kT) void plan_scan_tiles_kernel(int32_t* __restrict__ tilesum, int64_t ntiles,
                                                             unsigned long long* __restrict__ stat,
                                                             int32_t* __restrict__ rowptr_s,
                                                             int32_t* __restrict__ multi_first,
                                                             int64_t max_multi_rows) {
  __shared__ int wsum[kT / 64];
  __shared__ long long totals[5];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int c = 0; c < 5; ++c) {
    int32_t* __restrict__ ts = tilesum + (int64_t)c * (ntiles + 1);
    long long carry = 0;
    for (int64_t base = 0; base < ntiles; base += kRowTile) {
      const int64_t i0 = base + (int64_t)threadIdx.x * 8;
      int x[8], sum = 0;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        x[i] = (i0 + i < ntiles) ? ts[i0 + i] : 0;
        sum += x[i];
      }
      int inc = sum;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const int t = __shfl_up(inc, d, 64);
        if (lane >= d) inc += t;
      }
      if (lane == 63) wsum[wave] = inc;
      __syncthreads();
      int before = 0, total = 0;
#pragma unroll
      for (int w = 0; w < kT / 64; ++w) {
        if (w < wave) before += wsum[w];
        total += wsum[w];
      }
      __syncthreads();
      long long run = carry + before + inc - sum;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (i0 + i < ntiles) ts[i0 + i] = (int32_t)run;
        run += x[i];
      }
      carry += total;
    }
    if (threadIdx.x == 0) totals[c] = carry;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int c = 0; c < 5; ++c) stat[ST_PIECES + c] = (unsigned long long)totals[c];
    rowptr_s[totals[1]] = (int32_t)totals[2];
    if (totals[3] <= max_multi_rows) multi_first[totals[3]] = (int32_t)totals[4];
  }
}

// entries of the pieces of every window (a window = `window` consecutive pieces in row order)
__global__ __launch_bounds__(kT) void plan_window_entries_kernel(const int32_t* __restrict__ size, int64_t P,
                                                                 int64_t window,
                                                                 unsigned long long* __restrict__ win_entries) {
  const int64_t stride = (int64_t)gridDim.x * kT;
  for (int64_t base = (int64_t)blockIdx.x * kT; base < P; base += stride) {
    const int64_t id = base + threadIdx.x;
    const bool act = id < P;
    long long v = act ? size[id] : 0;
    const int64_t w = (act ? id : P - 1) / window;
    const int64_t w0 = __shfl(w, 0, 64), w63 = __shfl(w, 63, 64);
    if (w0 == w63) {        // the whole wavefront is inside one window: one atomic
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
      if ((threadIdx.x & 63) == 0 && v) atomicAdd(&win_entries[w0], (unsigned long long)v);
    } else if (act) {
      atomicAdd(&win_entries[w], (unsigned long long)v);
    }
  }
}

__global__ __launch_bounds__(kT) void plan_piece_keys_kernel(const int32_t* __restrict__ size, int64_t P,
                                                             int64_t window, uint32_t* __restrict__ keys) {
  const int64_t stride = (int64_t)gridDim.x * kT;
  for (int64_t id = (int64_t)blockIdx.x * kT + threadIdx.x; id < P; id += stride)
    keys[id] = ((uint32_t)(id / window) << 15) | (uint32_t)(32768 - size[id]);
}

__global__ __launch_bounds__(kT) void plan_fill_tables_kernel(int32_t* __restrict__ info, int32_t* __restrict__ target,
                                                              int64_t n_slots) {
  const int64_t stride = (int64_t)gridDim.x * kT;
  for (int64_t g = (int64_t)blockIdx.x * kT + threadIdx.x; g < n_slots; g += stride) {
    info[2 * g] = -1;
    info[2 * g + 1] = -1;
    target[g] = INT32_MIN;
  }
}

__global__ __launch_bounds__(kT) void plan_zero_units_kernel(int32_t* __restrict__ load, int32_t* __restrict__ used,
                                                             int64_t U, int32_t* __restrict__ done,
                                                             int32_t* __restrict__ assigned, int32_t nwin) {
  const int64_t stride = (int64_t)gridDim.x * kT;
  for (int64_t u = (int64_t)blockIdx.x * kT + threadIdx.x; u < U; u += stride) {
    load[u] = 0;
    used[u] = 0;
  }
  if (blockIdx.x == 0)
    for (int w = threadIdx.x; w < nwin; w += kT) {
      done[w] = 0;
      assigned[w] = 0;
    }
}

struct DealDims {
  int64_t P, window, U;    // pieces, pieces per window, streams (units) in all
  int32_t nwin, R, SL;     // windows, lane groups per wavefront, slots per unit
};

__device__ __forceinline__ int32_t window_of_unit(const int32_t* __restrict__ win_unit0, int32_t nwin, int64_t u) {
  int32_t lo = 0, hi = nwin;   // win_unit0[lo] <= u < win_unit0[hi]
  while (hi - lo > 1) {
    const int32_t mid = (lo + hi) >> 1;
    if ((int64_t)win_unit0[mid] <= u) lo = mid; else hi = mid;
  }
  return lo;
}

__device__ __forceinline__ int64_t window_pieces(const DealDims& d, int32_t w) {
  const int64_t a = (int64_t)w * d.window;
  return (a + d.window < d.P ? a + d.window : d.P) - a;
}

__device__ __forceinline__ void put_piece(int32_t* __restrict__ info, int32_t* __restrict__ target, int64_t g,
                                          const PieceArrays& pa, int64_t id) {
  const int32_t row = pa.row[id], mf = pa.mf[id];
  info[2 * g] = row;
  info[2 * g + 1] = pa.jp[id];
  target[g] = mf < 0 ? row : -mf - 1;
}

// sort key of a stream: (window, length) while it has a free slot and its window has pieces left
__global__ __launch_bounds__(kT) void deal_keys_kernel(DealDims d, const int32_t* __restrict__ win_unit0,
                                                       const int32_t* __restrict__ load,
                                                       const int32_t* __restrict__ used,
                                                       const int32_t* __restrict__ done,
                                                       uint32_t* __restrict__ keys) {
  const int64_t stride = (int64_t)gridDim.x * kT;
  for (int64_t u = (int64_t)blockIdx.x * kT + threadIdx.x; u < d.U; u += stride) {
    const int32_t w = window_of_unit(win_unit0, d.nwin, u);
    const bool open = used[u] < d.SL && (int64_t)done[w] < window_pieces(d, w);
    keys[u] = open ? (((uint32_t)w << 20) | (uint32_t)load[u]) : kFullUnit;
  }
}

// first[w] = first position of window w in the sorted stream keys (several windows only)
__global__ __launch_bounds__(kT) void deal_first_kernel(DealDims d, const uint32_t* __restrict__ skeys,
                                                        int32_t* __restrict__ first) {
  const int w = blockIdx.x * kT + threadIdx.x;
  if (w >= d.nwin) return;
  const uint32_t wkey = (uint32_t)w << 20;
  int64_t lo = 0, hi = d.U;
  while (lo < hi) {
    const int64_t mid = (lo + hi) >> 1;
    if (skeys[mid] < wkey) lo = mid + 1; else hi = mid;
  }
  first[w] = (int32_t)lo;
}

// position i of the sorted streams: the rank-th shortest open stream of its window takes the
// rank-th largest piece the window has left, for rank < B = half the window's streams
__global__ __launch_bounds__(kT) void deal_assign_kernel(DealDims d, const int32_t* __restrict__ win_unit0,
                                                         const uint32_t* __restrict__ skeys,
                                                         const uint32_t* __restrict__ sunit,
                                                         const int32_t* __restrict__ first,
                                                         const uint32_t* __restrict__ piece_order, PieceArrays pa,
                                                         int32_t* __restrict__ load, int32_t* __restrict__ used,
                                                         const int32_t* __restrict__ done,
                                                         int32_t* __restrict__ assigned, int32_t* __restrict__ info,
                                                         int32_t* __restrict__ target) {
  const int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i >= d.U) return;
  const uint32_t key = skeys[i];
  if (key == kFullUnit) return;
  const int32_t w = (int32_t)(key >> 20);
  if (w >= d.nwin) return;
  const int64_t rank = i - (d.nwin > 1 ? (int64_t)first[w] : 0);
  const int64_t units_w = (int64_t)win_unit0[w + 1] - win_unit0[w];
  const int64_t B = units_w / 2 > 0 ? units_w / 2 : 1;
  const int64_t left = window_pieces(d, w) - done[w];
  if (rank >= B || rank >= left) return;
  const int64_t id = piece_order[(int64_t)w * d.window + done[w] + rank];
  const int64_t u = sunit[i];
  const int32_t slot = used[u];
  used[u] = slot + 1;
  load[u] += pa.size[id];
  put_piece(info, target, (u / d.R) * kSweepSlots + (u % d.R) * d.SL + slot, pa, id);
  atomicAdd(&assigned[w], 1);
}

__global__ __launch_bounds__(kT) void deal_advance_kernel(int32_t* __restrict__ done, int32_t* __restrict__ assigned,
                                                          int32_t nwin) {
  const int w = blockIdx.x * kT + threadIdx.x;
  if (w < nwin) {
    done[w] += assigned[w];
    assigned[w] = 0;
  }
}

// flag[0] = 1 if a window still has pieces, else 0 (one workgroup)
__global__ __launch_bounds__(kT) void deal_check_kernel(DealDims d, const int32_t* __restrict__ done,
                                                        int32_t* __restrict__ flag) {
  __shared__ int any;
  if (threadIdx.x == 0) any = 0;
  __syncthreads();
  for (int w = threadIdx.x; w < d.nwin; w += kT)
    if ((int64_t)done[w] != window_pieces(d, w)) any = 1;
  __syncthreads();
  if (threadIdx.x == 0) flag[0] = any;
}

// Snake dealing (one row per instruction only, an experiment option): slot by slot across the
// window's wavefronts, alternating direction.
__global__ __launch_bounds__(kT) void deal_snake_kernel(DealDims d, const int32_t* __restrict__ win_unit0,
                                                        const uint32_t* __restrict__ piece_order, PieceArrays pa,
                                                        int32_t* __restrict__ info, int32_t* __restrict__ target,
                                                        int32_t* __restrict__ flag) {
  const int64_t stride = (int64_t)gridDim.x * kT;
  for (int64_t t = (int64_t)blockIdx.x * kT + threadIdx.x; t < d.P; t += stride) {
    const int64_t w = t / d.window, tw = t - w * d.window;
    const int64_t nw = (int64_t)win_unit0[w + 1] - win_unit0[w];
    const int64_t slot = tw / nw, pos = tw % nw;
    if (slot >= d.SL) { flag[0] = 1; continue; }
    const int64_t wv = win_unit0[w] + ((slot & 1) ? nw - 1 - pos : pos);
    put_piece(info, target, wv * kSweepSlots + slot, pa, piece_order[t]);
  }
}

// Short rows as whole-row pieces: sorted by length (descending, row order inside a length), 16
// consecutive ones per wavefront, so the rows of a wavefront -- and with lane groups the rows of
// its groups -- have nearly the same length.
__global__ __launch_bounds__(kT) void short_keys_kernel(const int32_t* __restrict__ size, int64_t n,
                                                        uint32_t* __restrict__ keys) {
  const int64_t stride = (int64_t)gridDim.x * kT;
  for (int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x; i < n; i += stride) {
    const int32_t d = size[i];
    keys[i] = (uint32_t)(255 - (d > 255 ? 255 : (d < 0 ? 0 : d)));
  }
}

__global__ __launch_bounds__(kT) void deal_short_kernel(const uint32_t* __restrict__ order, int64_t n, int64_t id0,
                                                        int64_t slot0, PieceArrays pa, int32_t* __restrict__ info,
                                                        int32_t* __restrict__ target) {
  const int64_t stride = (int64_t)gridDim.x * kT;
  for (int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x; i < n; i += stride)
    put_piece(info, target, slot0 + i, pa, id0 + (int64_t)order[i]);
}

struct PlanScratch {
  PieceArrays pa;
  uint32_t* piece_keys;
  uint32_t* unit_keys;
  int32_t *load, *used;
  RadixWs radix;
  size_t bytes;
};

PlanScratch carve_plan(char* base, int64_t max_pieces, int64_t max_units) {
  PlanScratch p{};
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char* q = base ? base + off : nullptr;
    off += round_up(bytes, 256);
    return q;
  };
  const size_t pw = sizeof(int32_t) * (size_t)max_pieces, uw = sizeof(int32_t) * (size_t)max_units;
  p.pa.row = reinterpret_cast<int32_t*>(take(pw));
  p.pa.jp = reinterpret_cast<int32_t*>(take(pw));
  p.pa.size = reinterpret_cast<int32_t*>(take(pw));
  p.pa.mf = reinterpret_cast<int32_t*>(take(pw));
  p.piece_keys = reinterpret_cast<uint32_t*>(take(pw));
  p.unit_keys = reinterpret_cast<uint32_t*>(take(uw));
  p.load = reinterpret_cast<int32_t*>(take(uw));
  p.used = reinterpret_cast<int32_t*>(take(uw));
  // the piece order (payload of the piece sort) must survive the stream sorts: two workspaces
  p.radix = carve_radix(base ? base + off : nullptr, std::max(max_pieces, max_units));
  off += p.radix.bytes;
  p.bytes = off;
  return p;
}

struct PlanSmall {               // the L.plan region
  unsigned long long* stat;      // [ST_COUNT]
  unsigned long long* win_entries;  // [kSweepMaxWindows]
  int32_t *win_unit0, *done, *assigned;   // [kSweepMaxWindows + 1] each
  int32_t* tilesum;              // [5][ntiles + 1]
};

PlanSmall carve_small(char* ws, const SpmmWsLayout& L) {
  PlanSmall p{};
  char* b = ws + L.plan;
  p.stat = reinterpret_cast<unsigned long long*>(b); b += 256;
  p.win_entries = reinterpret_cast<unsigned long long*>(b); b += 8 * (size_t)kSweepMaxWindows;
  p.win_unit0 = reinterpret_cast<int32_t*>(b); b += 4 * (size_t)(kSweepMaxWindows + 64);
  p.done = reinterpret_cast<int32_t*>(b); b += 4 * (size_t)(kSweepMaxWindows + 64);
  p.assigned = reinterpret_cast<int32_t*>(b); b += 4 * (size_t)(kSweepMaxWindows + 64);
  p.tilesum = reinterpret_cast<int32_t*>(b);
  return p;
}

dim3 grid_for(int64_t items) {
  int64_t b = ceil_div(items > 0 ? items : 1, kT);
  if (b > 256 * 16) b = 256 * 16;
  return dim3((unsigned)b);
}

}  // namespace

bool sweep_plan_fits(const SpmmWsLayout& L) {
  const size_t have = L.piece_info - L.code;     // the stream arrays, unused until the build pass
  return carve_plan(nullptr, L.max_pieces, L.max_waves * kSweepSlots).bytes <= have;
}

int sweep_plan_rows(const int32_t* d_rowptr, int64_t m, int64_t nnz, int32_t opt_min_long, int32_t piece_max,
                    char* ws, const SpmmWsLayout& L, hipStream_t s, SweepRowTotals* out, bool short_pieces) {
  const PlanSmall sm = carve_small(ws, L);
  const PlanScratch sc = carve_plan(ws + L.code, L.max_pieces, L.max_waves * kSweepSlots);
  int32_t* d_flag = reinterpret_cast<int32_t*>(ws + L.carry);
  const int64_t ntiles = ceil_div(m, kRowTile);
  hipLaunchKernelGGL(plan_zero_kernel, dim3(1), dim3(kT), 0, s, sm.stat, d_flag);
  SAGNN_LAUNCH_CHECK();
  hipLaunchKernelGGL(plan_rowstat_kernel, grid_for(m), dim3(kT), 0, s, d_rowptr, m, nnz, sm.stat);
  SAGNN_LAUNCH_CHECK();
  hipLaunchKernelGGL(plan_rule_kernel, dim3(1), dim3(64), 0, s, sm.stat, nnz, opt_min_long);
  SAGNN_LAUNCH_CHECK();
  int32_t* rowptr_s = reinterpret_cast<int32_t*>(ws + L.rowptr_s);
  int32_t* rowmap_s = reinterpret_cast<int32_t*>(ws + L.rowmap_s);
  int32_t* multi_row = reinterpret_cast<int32_t*>(ws + L.multi_row);
  int32_t* multi_first = reinterpret_cast<int32_t*>(ws + L.multi_first);
  hipLaunchKernelGGL(plan_rows_kernel<false>, dim3((unsigned)ntiles), dim3(kT), 0, s, d_rowptr, m, piece_max, ntiles,
                     sm.stat, sm.tilesum, rowptr_s, rowmap_s, multi_row, multi_first, sc.pa, L.max_pieces,
                     L.max_multi_rows, 0);
  SAGNN_LAUNCH_CHECK();
  hipLaunchKernelGGL(plan_scan_tiles_kernel, dim3(1), dim3(kT), 0, s, sm.tilesum, ntiles, sm.stat, rowptr_s,
                     multi_first, L.max_multi_rows);
  SAGNN_LAUNCH_CHECK();
  hipLaunchKernelGGL(plan_rows_kernel<true>, dim3((unsigned)ntiles), dim3(kT), 0, s, d_rowptr, m, piece_max, ntiles,
                     sm.stat, sm.tilesum, rowptr_s, rowmap_s, multi_row, multi_first, sc.pa, L.max_pieces,
                     L.max_multi_rows, short_pieces ? 1 : 0);
  SAGNN_LAUNCH_CHECK();
  unsigned long long h[ST_COUNT];
  SAGNN_HIP(hipMemcpyAsync(h, sm.stat, sizeof(h), hipMemcpyDeviceToHost, s));
  SAGNN_HIP(hipStreamSynchronize(s));
  out->bad = h[ST_BAD] != 0;
  out->has_empty = h[ST_EMPTY] != 0;
  out->min_long = (int32_t)h[ST_MINLONG];
  out->pieces = (int64_t)h[ST_PIECES];
  out->short_rows = (int64_t)h[ST_SHORT_ROWS];
  out->short_entries = (int64_t)h[ST_SHORT_ENTRIES];
  out->multi_rows = (int64_t)h[ST_MULTI_ROWS];
  out->multi_pieces = (int64_t)h[ST_MULTI_PIECES];
  return SAGNN_OK;
}

int sweep_plan_window_entries(char* ws, const SpmmWsLayout& L, int64_t P, int64_t window, int32_t nwin,
                              hipStream_t s, std::vector<int64_t>* entries) {
  const PlanSmall sm = carve_small(ws, L);
  const PlanScratch sc = carve_plan(ws + L.code, L.max_pieces, L.max_waves * kSweepSlots);
  SAGNN_HIP(hipMemsetAsync(sm.win_entries, 0, sizeof(unsigned long long) * (size_t)nwin, s));
  hipLaunchKernelGGL(plan_window_entries_kernel, grid_for(P), dim3(kT), 0, s, sc.pa.size, P, window, sm.win_entries);
  SAGNN_LAUNCH_CHECK();
  std::vector<unsigned long long> h((size_t)nwin);
  SAGNN_HIP(hipMemcpyAsync(h.data(), sm.win_entries, sizeof(unsigned long long) * (size_t)nwin,
                           hipMemcpyDeviceToHost, s));
  SAGNN_HIP(hipStreamSynchronize(s));
  entries->assign(h.begin(), h.end());
  return SAGNN_OK;
}

int sweep_plan_deal_short(char* ws, const SpmmWsLayout& L, int64_t P_long, int64_t n_short, int64_t first_wave,
                          hipStream_t s) {
  const PlanScratch sc = carve_plan(ws + L.code, L.max_pieces, L.max_waves * kSweepSlots);
  int32_t* info = reinterpret_cast<int32_t*>(ws + L.piece_info);
  int32_t* target = reinterpret_cast<int32_t*>(ws + L.piece_target);
  if (n_short <= 0) return SAGNN_OK;
  if (P_long < 0 || P_long + n_short > L.max_pieces ||
      first_wave + ceil_div(n_short, (int64_t)kSweepSlots) > L.max_waves)
    return SAGNN_EINVAL;
  // the key array of the pieces is free once the long pieces have been dealt (stream order)
  hipLaunchKernelGGL(short_keys_kernel, grid_for(n_short), dim3(kT), 0, s, sc.pa.size + P_long, n_short,
                     sc.piece_keys);
  SAGNN_LAUNCH_CHECK();
  int res = 0;
  const int rc = radix_sort_pairs(sc.piece_keys, nullptr, n_short, 8, sc.radix, s, &res);
  if (rc != SAGNN_OK) return rc;
  hipLaunchKernelGGL(deal_short_kernel, grid_for(n_short), dim3(kT), 0, s, sc.radix.pay[res], n_short, P_long,
                     first_wave * kSweepSlots, sc.pa, info, target);
  SAGNN_LAUNCH_CHECK();
  return SAGNN_OK;
}

int sweep_plan_deal(char* ws, const SpmmWsLayout& L, int64_t P, int64_t window, const int32_t* h_win_unit0,
                    int32_t nwin, int64_t n_waves4, int32_t R, int32_t SL, bool snake, hipStream_t s) {
  const PlanSmall sm = carve_small(ws, L);
  const PlanScratch sc = carve_plan(ws + L.code, L.max_pieces, L.max_waves * kSweepSlots);
  int32_t* d_flag = reinterpret_cast<int32_t*>(ws + L.carry);
  int32_t* info = reinterpret_cast<int32_t*>(ws + L.piece_info);
  int32_t* target = reinterpret_cast<int32_t*>(ws + L.piece_target);
  const int64_t U = h_win_unit0[nwin];
  if (nwin < 1 || nwin > kSweepMaxWindows || U < 1 || U > L.max_waves * kSweepSlots || P > L.max_pieces)
    return SAGNN_EINVAL;
  // the caller keeps h_win_unit0 alive until its next synchronisation
  SAGNN_HIP(hipMemcpyAsync(sm.win_unit0, h_win_unit0, sizeof(int32_t) * (size_t)(nwin + 1), hipMemcpyHostToDevice, s));
  hipLaunchKernelGGL(plan_fill_tables_kernel, grid_for(n_waves4 * kSweepSlots), dim3(kT), 0, s, info, target,
                     n_waves4 * kSweepSlots);
  SAGNN_LAUNCH_CHECK();

  // pieces by (window, size descending); ties keep the row order
  hipLaunchKernelGGL(plan_piece_keys_kernel, grid_for(P), dim3(kT), 0, s, sc.pa.size, P, window, sc.piece_keys);
  SAGNN_LAUNCH_CHECK();
  int wbits = 0;
  while ((1 << wbits) < nwin) ++wbits;
  int res = 0;
  int rc = radix_sort_pairs(sc.piece_keys, nullptr, P, 15 + wbits, sc.radix, s, &res);
  if (rc != SAGNN_OK) return rc;
  // keep the piece order where the stream sorts do not write: the key array of the pieces is free now
  uint32_t* piece_order = sc.piece_keys;
  SAGNN_HIP(hipMemcpyAsync(piece_order, sc.radix.pay[res], sizeof(uint32_t) * (size_t)P, hipMemcpyDeviceToDevice, s));

  DealDims d{P, window, U, nwin, R, SL};
  if (snake) {
    hipLaunchKernelGGL(deal_snake_kernel, grid_for(P), dim3(kT), 0, s, d, sm.win_unit0, piece_order, sc.pa, info,
                       target, d_flag + 2);
    SAGNN_LAUNCH_CHECK();
    return SAGNN_OK;
  }
  hipLaunchKernelGGL(plan_zero_units_kernel, grid_for(U), dim3(kT), 0, s, sc.load, sc.used, U, sm.done, sm.assigned,
                     nwin);
  SAGNN_LAUNCH_CHECK();
  // A stream has a free slot in at most SL batches after the batches of B pieces have ended, and
  // there are at most 2 SL + 1 of those: 3 SL + 2 batches deal every piece.  Usually the batches
  // of B pieces are enough, so after those the host looks every few batches whether pieces are left.
  const int max_batches = 3 * SL + 2;
  int64_t per_unit = 1;
  for (int32_t w = 0; w < nwin; ++w) {
    const int64_t a = (int64_t)w * window, n_w = std::min(P, a + window) - a;
    const int64_t units_w = (int64_t)h_win_unit0[w + 1] - h_win_unit0[w];
    per_unit = std::max(per_unit, ceil_div(n_w, std::max<int64_t>(units_w / 2, 1)));
  }
  int next_check = (int)std::min<int64_t>(per_unit + 1, max_batches);
  for (int b = 0; b < max_batches; ++b) {
    hipLaunchKernelGGL(deal_keys_kernel, grid_for(U), dim3(kT), 0, s, d, sm.win_unit0, sc.load, sc.used, sm.done,
                       sc.unit_keys);
    SAGNN_LAUNCH_CHECK();
    rc = radix_sort_pairs(sc.unit_keys, nullptr, U, nwin > 1 ? 20 + wbits : 24, sc.radix, s, &res);
    if (rc != SAGNN_OK) return rc;
    int32_t* first = reinterpret_cast<int32_t*>(sm.win_entries);   // the window sums have been read back
    if (nwin > 1) {
      hipLaunchKernelGGL(deal_first_kernel, dim3((unsigned)ceil_div(nwin, kT)), dim3(kT), 0, s, d,
                         sc.radix.keys[res], first);
      SAGNN_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(deal_assign_kernel, dim3((unsigned)ceil_div(U, kT)), dim3(kT), 0, s, d, sm.win_unit0,
                       sc.radix.keys[res], sc.radix.pay[res], first, piece_order, sc.pa, sc.load, sc.used, sm.done,
                       sm.assigned, info, target);
    SAGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(deal_advance_kernel, dim3((unsigned)ceil_div(nwin, kT)), dim3(kT), 0, s, sm.done, sm.assigned,
                       nwin);
    SAGNN_LAUNCH_CHECK();
    if (b + 1 == next_check || b + 1 == max_batches) {
      hipLaunchKernelGGL(deal_check_kernel, dim3(1), dim3(kT), 0, s, d, sm.done, d_flag + 2);
      SAGNN_LAUNCH_CHECK();
      int32_t left = 0;
      SAGNN_HIP(hipMemcpyAsync(&left, d_flag + 2, sizeof(int32_t), hipMemcpyDeviceToHost, s));
      SAGNN_HIP(hipStreamSynchronize(s));
      if (!left) break;
      next_check = b + 1 + 3;
    }
  }
  return SAGNN_OK;
}

}  // namespace sagnn
