// Locality-aware schedule for the local SpMM of power-law graphs: the "slab sweep".
//
// Why: in C = A * B (Alg. 1 / Alg. 2, "Z <- Z + SpMM(A_iq, H^)") every stored entry pulls one
// f-wide row of B through the memory system.  With a randomly ordered power-law graph a row of
// B is almost never still in a 4 MB per-XCD L2 when it is needed again, so the plain schedule
// moves ~15x the compulsory bytes over the fabric (measured).  The paper fixes the sparsity
// pattern for the whole training run (it partitions once and reuses the plan every epoch), so
// a one-time re-ordering of the entry stream is free to choose WHEN each row of B is touched.
//
// What: the rows of B are cut into S contiguous slabs.  Rows of A with at least `min_long`
// entries ("long" rows; they hold most entries of a power-law graph) are cut into pieces of at
// most `piece_max` entries, and every wavefront is given kSweepSlots pieces whose entries it
// walks slab by slab: all entries that reference slab 0, then slab 1, ...  Because all resident
// wavefronts walk the slabs in the same order at about the same pace (their streams have nearly
// equal lengths), each XCD's L2 only has to hold the hot rows of ONE slab at a time, and a slab
// that one XCD has pulled from HBM is served to the other seven from the memory-side cache.
// (Starting the XCDs at different slabs was measured to be slower: it defeats that sharing.)
// Per-piece accumulators live in LDS (a wavefront adds its register accumulator to the piece's
// LDS row whenever a (piece, slab) segment ends), so nothing is spilled to HBM between slabs.
// Pieces of a split row are summed in a fixed order by a small second kernel.  Short rows are
// swept as whole rows -- 16 per wavefront, each one segment, in wavefronts of their own -- where
// the matrix allows it, else they go through the nonzero-splitting kernels of spmm.hip on a
// compacted CSR.
//
// The entry stream of a wavefront is stored in the workspace as (code, value) pairs sorted by
// (slab, piece): code = column | piece_slot << 27 | segment_end << 31.  At f = 128 / 64 a
// wavefront can carry 2 / 4 such streams, one per lane group, stored zipped (see
// spmm_sweep_group_kernel): a group of 32 / 16 lanes moves a whole row of B, so one load
// instruction serves 2 / 4 entries.
#include <stdlib.h>

#include <algorithm>
#include <atomic>
#include <functional>
#include <vector>

#include "common.h"
#include "rowload.h"

namespace sagnn {
namespace {

constexpr int kBuildThreads = 256;
constexpr uint32_t kColMask = (1u << kSweepColBits) - 1u;

// ---------------------------------------------------------------------------------------
// preparation kernels

// piece_info[2*g] = row (or -1), piece_info[2*g+1] = (j << 16) | p.  One wavefront per piece
// slot with j == 0 checks that its row's column indices are ascending and inside [0, k).
__global__ __launch_bounds__(256) void sweep_check_sorted_kernel(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
    const int32_t* __restrict__ piece_info, int64_t n_slots, uint32_t kmax,
    int32_t* __restrict__ unsorted) {
  const int lane = threadIdx.x & 63;
  const int64_t g = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6;
  if (g >= n_slots) return;
  const int32_t row = piece_info[2 * g];
  if (row < 0 || (piece_info[2 * g + 1] >> 16) != 0) return;
  const int32_t b = rowptr[row], e = rowptr[row + 1];
  bool bad = false;
  for (int32_t i = b + lane; i < e; i += 64) {
    bad |= (uint32_t)colidx[i] > kmax;                       // negative or >= k
    if (i + 1 < e) bad |= colidx[i] > colidx[i + 1];
  }
  if (bad) *unsorted = 1;
}

__device__ __forceinline__ int32_t count_upto(int32_t x, int32_t j, int32_t p) {
  // number of i in [0, x) with i % p == j
  return x > j ? (x - j + p - 1) / p : 0;
}

// Per-wavefront segment tables shared by the counting and the building kernel (dynamic LDS):
//   lo[16][S+1]      first entry (index in its row) of slab s for the piece in a slot
//   off[S][16]       offset of segment (s, slot) inside its slab, per lane group
//   slab_tot[S][16]  entries of slab s per lane group
struct BuildTables {
  int32_t *lo, *off, *slab_tot;
  int SS;
  __device__ int32_t& LO(int slot, int s) const { return lo[slot * (SS + 1) + s]; }
  __device__ int32_t& OFF(int s, int slot) const { return off[s * kSweepSlots + slot]; }
  __device__ int32_t& TOT(int s, int g) const { return slab_tot[s * kSweepSlots + g]; }
};

struct BuildPieces {
  int32_t row[kSweepSlots], j[kSweepSlots], p[kSweepSlots], beg[kSweepSlots], deg[kSweepSlots];
};

// fills pc (shared) and the tables for wavefront w; all threads of the workgroup take part
__device__ __forceinline__ void build_tables(const int32_t* __restrict__ rowptr,
                                             const int32_t* __restrict__ colidx,
                                             const int32_t* __restrict__ piece_info, int64_t w, int S,
                                             int32_t slab_width, uint32_t kmax, int R, int SL,
                                             BuildPieces& pc, const BuildTables& T) {
  const int tid = threadIdx.x;
  if (tid < kSweepSlots) {
    const int32_t row = piece_info[2 * (w * kSweepSlots + tid)];
    const int32_t jp = piece_info[2 * (w * kSweepSlots + tid) + 1];
    pc.row[tid] = row;
    pc.j[tid] = jp >> 16;
    pc.p[tid] = jp & 0xFFFF;
    pc.beg[tid] = row >= 0 ? rowptr[row] : 0;
    pc.deg[tid] = row >= 0 ? rowptr[row + 1] - rowptr[row] : 0;
  }
  __syncthreads();
  for (int idx = tid; idx < kSweepSlots * (S + 1); idx += kBuildThreads) {
    const int slot = idx / (S + 1), s = idx - slot * (S + 1);
    int32_t res = 0;
    if (pc.row[slot] >= 0) {
      const int32_t d = pc.deg[slot];
      if (s == S) {
        res = d;
      } else {
        // lower bound of column s*slab_width in the (ascending) row
        const int64_t target = (int64_t)s * slab_width;
        const int32_t* __restrict__ c = colidx + pc.beg[slot];
        int32_t a = 0, b = d;
        while (a < b) {
          const int32_t mid = (a + b) >> 1;
          const uint32_t cv = (uint32_t)c[mid] > kmax ? kmax : (uint32_t)c[mid];
          if ((int64_t)cv < target) a = mid + 1; else b = mid;
        }
        res = a;
      }
    }
    T.LO(slot, s) = res;
  }
  __syncthreads();
  // entries of segment (s, slot); then per slab the prefix over the slots of each group
  for (int idx = tid; idx < S * kSweepSlots; idx += kBuildThreads) {
    const int s = idx / kSweepSlots, slot = idx - s * kSweepSlots;
    T.OFF(s, slot) = pc.row[slot] >= 0 ? count_upto(T.LO(slot, s + 1), pc.j[slot], pc.p[slot]) -
                                             count_upto(T.LO(slot, s), pc.j[slot], pc.p[slot])
                                       : 0;
  }
  __syncthreads();
  for (int idx = tid; idx < S * R; idx += kBuildThreads) {
    const int s = idx / R, gi = idx - s * R;
    int32_t run = 0;
    for (int slot = gi * SL; slot < (gi + 1) * SL; ++slot) {
      const int32_t c = T.OFF(s, slot);
      T.OFF(s, slot) = run;
      run += c;
    }
    T.TOT(s, gi) = run;
  }
  __syncthreads();
}

__device__ __forceinline__ BuildTables carve_tables(int32_t* lds, int S) {
  BuildTables T;
  T.SS = S;
  T.lo = lds;
  T.off = T.lo + kSweepSlots * (S + 1);
  T.slab_tot = T.off + S * kSweepSlots;
  return T;
}

// Pass 1: length of every interval of a wavefront's stream.  An interval's R group streams are
// padded to the longest of them and to a whole batch (8 steps), so that every wavefront reaches
// an interval boundary at a batch boundary.  sync_off[w][i] = first step of interval i,
// wave_steps[w] = total steps.
__global__ __launch_bounds__(kBuildThreads) void sweep_count_kernel(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
    const int32_t* __restrict__ piece_info, int32_t n_slabs, int32_t slab_width, uint32_t kmax,
    int32_t groups, int32_t slots_per_group, int32_t n_intervals, int32_t sync_slabs,
    int32_t* __restrict__ sync_off, int32_t* __restrict__ wave_steps, int64_t first_whole_row_wave) {
  extern __shared__ __attribute__((aligned(16))) int32_t build_lds[];
  __shared__ BuildPieces pc;
  __shared__ int32_t ivl_len[kSweepMaxIntervals];
  const int64_t w = blockIdx.x;
  // wavefronts of whole short rows keep every row as one segment: one slab that covers all of B
  if (w >= first_whole_row_wave) {
    n_slabs = 1;
    slab_width = 0x7FFFFFFF;
  }
  const int S = n_slabs, R = groups;
  const BuildTables T = carve_tables(build_lds, S);
  build_tables(rowptr, colidx, piece_info, w, S, slab_width, kmax, R, slots_per_group, pc, T);
  const int per = sync_slabs > 0 ? sync_slabs : S;
  for (int i = threadIdx.x; i < n_intervals; i += kBuildThreads) {
    const int s0 = i * per, s1 = (i + 1) * per < S ? (i + 1) * per : S;
    int32_t longest = 0;
    for (int gi = 0; gi < R; ++gi) {
      int32_t t = 0;
      for (int s = s0; s < s1; ++s) t += T.TOT(s, gi);
      longest = t > longest ? t : longest;
    }
    ivl_len[i] = (longest + 7) & ~7;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int32_t run = 0;
    int32_t* so = sync_off + w * (kSweepMaxIntervals + 1);
    for (int i = 0; i < n_intervals; ++i) {
      so[i] = run;
      run += ivl_len[i];
    }
    so[n_intervals] = run;
    wave_steps[w] = run;
  }
}

// Pass 2 (one workgroup): wave_base[w] = R * (steps of the wavefronts before w); wave_base[NW]
// is the total stream length.  overflow[0] = 1 if it does not fit 31 bits.
__global__ __launch_bounds__(1024) void sweep_scan_kernel(const int32_t* __restrict__ wave_steps,
                                                          int64_t n_waves, int32_t groups,
                                                          int32_t* __restrict__ wave_base,
                                                          int32_t* __restrict__ overflow) {
  __shared__ int64_t part[1024];
  const int tid = threadIdx.x;
  const int64_t per = (n_waves + 1023) / 1024;
  const int64_t a = tid * per, b = a + per < n_waves ? a + per : n_waves;
  int64_t sum = 0;
  for (int64_t w = a; w < b; ++w) sum += (int64_t)wave_steps[w] * groups;
  part[tid] = sum;
  __syncthreads();
  if (tid == 0) {
    int64_t run = 0;
    for (int i = 0; i < 1024; ++i) {
      const int64_t t = part[i];
      part[i] = run;
      run += t;
    }
    overflow[0] = run > 0x7FFFFFF0ll ? 1 : 0;
    wave_base[n_waves] = (int32_t)(run > 0x7FFFFFF0ll ? 0x7FFFFFF0ll : run);
  }
  __syncthreads();
  int64_t run = part[tid];
  for (int64_t w = a; w < b; ++w) {
    wave_base[w] = (int32_t)(run > 0x7FFFFFF0ll ? 0x7FFFFFF0ll : run);
    run += (int64_t)wave_steps[w] * groups;
  }
}

// Pass 3, one workgroup per wavefront: lay the entries out in (interval, slab, piece) order and
// encode them.  With `groups` = R lane groups the wavefront carries R independent streams (group
// g owns slots g*SL .. g*SL+SL-1), stored zipped: step t of group g at position R*t + g.  Steps that no
// entry lands on (padding of the shorter group streams and at interval boundaries) multiply
// row 0 of B by 0.
__global__ __launch_bounds__(kBuildThreads) void sweep_build_kernel(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
    const float* __restrict__ val, const int32_t* __restrict__ piece_info,
    const int32_t* __restrict__ wave_base, const int32_t* __restrict__ sync_off, int32_t n_slabs,
    int32_t slab_width, uint32_t kmax, int32_t groups, int32_t slots_per_group, int32_t n_intervals,
    int32_t sync_slabs, uint32_t* __restrict__ code, float* __restrict__ vals, int64_t first_whole_row_wave) {
  extern __shared__ __attribute__((aligned(16))) int32_t build_lds[];
  __shared__ BuildPieces pc;
  const int64_t w = blockIdx.x;
  const int tid = threadIdx.x;
  if (w >= first_whole_row_wave) {   // whole short rows: one segment per row (see sweep_count_kernel)
    n_slabs = 1;
    slab_width = 0x7FFFFFFF;
  }
  const int S = n_slabs, R = groups, SL = slots_per_group;
  const BuildTables T = carve_tables(build_lds, S);
  int32_t* slab_base_ = T.slab_tot + S * kSweepSlots;          // [S][16]: first step of slab s, group g
  build_tables(rowptr, colidx, piece_info, w, S, slab_width, kmax, R, SL, pc, T);
  const int per = sync_slabs > 0 ? sync_slabs : S;
  const int32_t* __restrict__ so = sync_off + w * (kSweepMaxIntervals + 1);
  for (int idx = tid; idx < n_intervals * R; idx += kBuildThreads) {
    const int i = idx / R, gi = idx - i * R;
    const int s0 = i * per, s1 = (i + 1) * per < S ? (i + 1) * per : S;
    int32_t run = so[i];
    for (int s = s0; s < s1; ++s) {
      slab_base_[s * kSweepSlots + gi] = run;
      run += T.TOT(s, gi);
    }
  }
  const int64_t base = wave_base[w];
  const int64_t words = (int64_t)so[n_intervals] * R;
  for (int64_t t = tid; t < words; t += kBuildThreads) {
    code[base + t] = 0u;
    vals[base + t] = 0.f;
  }
  __syncthreads();
  for (int slot = 0; slot < kSweepSlots; ++slot) {
    if (pc.row[slot] < 0) continue;
    const int gi = slot / SL;
    const int32_t j = pc.j[slot], p = pc.p[slot], d = pc.deg[slot], beg = pc.beg[slot];
    const int32_t size = count_upto(d, j, p);
    for (int32_t t = tid; t < size; t += kBuildThreads) {
      const int32_t i = j + t * p;
      const uint32_t craw = (uint32_t)colidx[beg + i];
      const uint32_t c = craw > kmax ? kmax : craw;
      int s = (int)(c / (uint32_t)slab_width);
      if (s > S - 1) s = S - 1;
      // the row is ascending, but clamped / equal columns may sit on a slab boundary: trust lo[]
      while (s > 0 && i < T.LO(slot, s)) --s;
      while (s < S - 1 && i >= T.LO(slot, s + 1)) ++s;
      const int32_t rank = t - count_upto(T.LO(slot, s), j, p);
      // a segment also ends every kSweepRunMax entries, which bounds the length of any serial
      // fp32 accumulation (and with it the rounding bias on rows of equal terms)
      const bool last = i + p >= T.LO(slot, s + 1) || (rank & (kSweepRunMax - 1)) == kSweepRunMax - 1;
      const int64_t pos = base + (int64_t)(slab_base_[s * kSweepSlots + gi] + T.OFF(s, slot) + rank) * R + gi;
      code[pos] = c | ((uint32_t)slot << kSweepColBits) | (last ? 0x80000000u : 0u);
      vals[pos] = val[beg + i];
    }
  }
}

inline size_t sweep_count_lds_bytes(int64_t S) {
  return sizeof(int32_t) * (size_t)(kSweepSlots * (S + 1) + 2 * S * kSweepSlots);
}
inline size_t sweep_build_lds_bytes(int64_t S) {
  return sizeof(int32_t) * (size_t)(kSweepSlots * (S + 1) + 3 * S * kSweepSlots);
}

__global__ __launch_bounds__(256) void sweep_zero_gap_kernel(uint32_t* __restrict__ code,
                                                            float* __restrict__ vals, int32_t n) {
  for (int i = threadIdx.x; i < n; i += 256) {
    code[i] = 0u;
    vals[i] = 0.f;
  }
}

// compacted CSR of the short rows: copy entries
__global__ __launch_bounds__(256) void sweep_short_copy_kernel(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
    const float* __restrict__ val, const int32_t* __restrict__ rowptr_s,
    const int32_t* __restrict__ rowmap_s, int64_t rows_s, int32_t* __restrict__ colidx_s,
    float* __restrict__ val_s) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= rows_s) return;
  const int32_t r = rowmap_s[i];
  const int32_t b = rowptr[r], n = rowptr[r + 1] - b, o = rowptr_s[i];
  for (int32_t t = 0; t < n; ++t) {
    colidx_s[o + t] = colidx[b + t];
    val_s[o + t] = val[b + t];
  }
}

// ---------------------------------------------------------------------------------------
// product kernel
struct SweepDims {
  int64_t n_waves, ldb, ldc, f_total;
  uint64_t generation;
  uint32_t b_bytes;     // bytes addressable from B + col0 (buffer-load variant)
  uint32_t row_bytes;   // ldb * 4
  int32_t col0, accumulate;
  // interval barriers (lane-group kernels): 0 intervals = walk the stream in one go
  int32_t n_intervals, wg_per_cohort, sync_timeout_ticks, sync_test_extra;
  int32_t slots;        // accumulator rows per wavefront (<= kSweepSlots)
  float pace_ticks;     // pacing: 100 MHz ticks per stream step (0: none)
};

// Barrier between two intervals of the sweep for the workgroups that run at the same time on
// one XCD ("cohort" c = workgroup index / wg_per_cohort, XCD = workgroup index mod 8: workgroups
// are handed to the XCDs round-robin).  It only paces the workgroups -- no data passes through
// it -- so that all of them read the same part of B at the same time and the XCD's L2 serves
// every row once.  The wait is bounded: after `timeout` ticks of the 100 MHz clock the waiter
// sets a flag that makes every later barrier of the launch fall through (the kernel then
// free-runs, correct but with more cache misses), so a launch whose cohort is not resident
// together (fewer free CUs than assumed) still ends.
__device__ __forceinline__ void sweep_interval_barrier(uint32_t* __restrict__ counters, int slot,
                                                       uint32_t expected, int32_t timeout) {
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t* broken = counters + kSweepBarrierSlots;
    if (__hip_atomic_load(broken, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) {
      uint32_t* ctr = counters + slot;
      __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const uint64_t t0 = wall_clock64();
      while (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < expected) {
        if (__hip_atomic_load(broken, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
        if (wall_clock64() - t0 > (uint64_t)timeout) {
          __hip_atomic_store(broken, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          break;
        }
        __builtin_amdgcn_s_sleep(16);
      }
    }
  }
  __syncthreads();
}

// Pacing: a wavefront does not enter the next interval before `ticks` of the 100 MHz clock have
// passed since it started.  Every wavefront follows the same schedule (the average number of
// stream steps up to each interval boundary, times a fixed time per step), so all of them pass
// over B at one pace without exchanging anything; one that is behind schedule never waits.  The
// loop is bounded (the clock passes the deadline, and the iteration count is capped anyway).
__device__ __forceinline__ void sweep_pace_until(uint64_t t0, float ticks) {
  const uint64_t deadline = t0 + (uint64_t)ticks;
  for (int i = 0; i < 2048; ++i) {
    if ((uint64_t)wall_clock64() >= deadline) break;
    __builtin_amdgcn_s_sleep(8);
  }
}

// sched[i] = average over the wavefronts of the first step of interval i (i = 0..n_intervals);
// sched[n_intervals + 1] = the longest stream (steps), written by one more workgroup
__global__ __launch_bounds__(256) void sweep_sched_kernel(const int32_t* __restrict__ sync_off,
                                                          int64_t n_waves, int32_t n_intervals,
                                                          float* __restrict__ sched) {
  __shared__ double red[256];
  const int i = blockIdx.x;
  const bool want_max = i == n_intervals + 1;
  const int col = want_max ? n_intervals : i;
  double acc = 0.0;
  for (int64_t w = threadIdx.x; w < n_waves; w += 256) {
    const double v = (double)sync_off[w * (kSweepMaxIntervals + 1) + col];
    acc = want_max ? (v > acc ? v : acc) : acc + v;
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int d = 128; d > 0; d >>= 1) {
    if ((int)threadIdx.x < d) {
      const double o = red[threadIdx.x + d];
      red[threadIdx.x] = want_max ? (o > red[threadIdx.x] ? o : red[threadIdx.x]) : red[threadIdx.x] + o;
    }
    __syncthreads();
  }
  if (threadIdx.x == 0 && i <= n_intervals + 1)
    sched[i] = want_max ? (float)red[0] : (n_waves > 0 ? (float)(red[0] / (double)n_waves) : 0.f);
}

__global__ __launch_bounds__(256) void sweep_barrier_clear_kernel(uint32_t* __restrict__ counters, int n) {
  for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += gridDim.x * 256) counters[i] = 0u;
  if (blockIdx.x == 0 && threadIdx.x == 0) counters[kSweepBarrierSlots] = 0u;
}

template <int FPL, int U, bool BUF>
__global__ __launch_bounds__(256) void spmm_sweep_kernel(
    const uint32_t* __restrict__ code, const float* __restrict__ vals,
    const int32_t* __restrict__ wave_base, const int32_t* __restrict__ piece_target,
    const SpmmWsHeader* __restrict__ hdr, const float* __restrict__ B, float* __restrict__ C,
    float* __restrict__ partial, const SweepDims d) {
  using vec = typename Vec<FPL>::T;
  extern __shared__ __attribute__((aligned(16))) float lds_acc[];  // [4 waves][d.slots][64*FPL]
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t loff = lane * (FPL * 4);
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int64_t w = (int64_t)blockIdx.x * 4 + wave;
  if (w >= d.n_waves) return;
  if (hdr->magic != kSpmmMagic || hdr->generation != d.generation || hdr->n_waves != d.n_waves ||
      hdr->groups != 1)
    return;
  constexpr int kRow = 64 * FPL;  // floats per accumulator row
  float* __restrict__ my = lds_acc + (size_t)wave * d.slots * kRow + lane * FPL;
  for (int s = 0; s < d.slots; ++s) *reinterpret_cast<vec*>(my + s * kRow) = vec(0.f);

  const int32_t base = wave_base[w];
  const int32_t len = wave_base[w + 1] - base;  // a multiple of U (padded when built)
  const uint32_t* __restrict__ cw = code + base;
  const float* __restrict__ vw = vals + base;
  const __amdgpu_buffer_rsrc_t rs = make_rsrc(B, d.b_bytes);

  vec acc = 0.f;
  for (int32_t e = 0; e < len; e += U) {
    uint32_t c[U];
    float v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      c[u] = cw[e + u];
      v[u] = vw[e + u];
    }
    vec h[U];
#pragma unroll
    for (int u = 0; u < U; ++u) h[u] = load_row<FPL, BUF>(rs, B, c[u] & kColMask, loff, d.row_bytes, d.ldb);
#pragma unroll
    for (int u = 0; u < U; ++u) asm volatile("" : "+v"(h[u]));
#pragma unroll
    for (int u = 0; u < U; ++u) {
      acc += v[u] * h[u];
      if (c[u] >> 31) {   // last entry of a (piece, slab) segment: fold into the piece's LDS row
        vec* p = reinterpret_cast<vec*>(my + ((c[u] >> kSweepColBits) & (kSweepSlots - 1)) * kRow);
        *p += acc;
        acc = 0.f;
      }
    }
  }

#pragma unroll 1
  for (int s = 0; s < d.slots; ++s) {
    const int32_t tgt = piece_target[w * kSweepSlots + s];
    if (tgt == INT32_MIN) continue;
    vec r = *reinterpret_cast<const vec*>(my + s * kRow);
    if (tgt >= 0) {
      vec* p = reinterpret_cast<vec*>(reinterpret_cast<char*>(C + (int64_t)tgt * d.ldc) + loff);
      if (d.accumulate) r += *p;
      *p = r;
    } else {
      const int64_t pi = -(int64_t)tgt - 1;
      *reinterpret_cast<vec*>(reinterpret_cast<char*>(partial + pi * d.f_total + d.col0) + loff) = r;
    }
  }
}

// The sweep with the layer's dense transform as its epilogue (Alg. 1: the SpMM statement followed
// by GEMM and the activation): when a workgroup's four wavefronts have walked their streams, its
// LDS holds 64 finished rows of T = A H (4 x 16 accumulator rows), which is two 32-row operand
// tiles of the matrix cores.  Wavefront (rt, half) multiplies row tile rt by the 32-column tiles
// half, half + 2, .. of W, read from global memory (W is small and stays in L2), and stores the
// rows of Z / sigma(Z) at the rows the pieces belong to.  Rows that are cut into several pieces
// (their partial rows go to `partial` as usual) and rows outside the sweep are left to a
// separate small kernel.  T itself goes to memory only if the caller wants it.
typedef float sweep_floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 sweep_bf16x8 __attribute__((ext_vector_type(8)));

// Dense transform of a sweep workgroup's 64 finished rows of T (LDS, [4 waves][16 slots][KROW]):
// wavefront (rt, half) multiplies row tile rt by the 32-column tiles half, half + 2, .. of W and
// stores the rows of Z / sigma(Z) at the rows the pieces belong to (slots that hold a piece of a
// split row, or nothing, are skipped).  Called by all four wavefronts after a workgroup barrier.
// MODE: the matrix-core operands, numbered like SAGNN_GEMM_*: 0 fp32, 1 rounded to bfloat16, 2 fp32
// as the exact sum of three bfloat16 terms with the six products down to 2^-16 of the leading one.
// |t2| <= 2^-8 |x| and |t3| <= 2^-16 |x|; both subtractions are exact.
__device__ __forceinline__ void sweep_split3(float x, __bf16& t1, __bf16& t2, __bf16& t3) {
  t1 = (__bf16)x;
  const float r = x - (float)t1;
  t2 = (__bf16)r;
  t3 = (__bf16)(r - (float)t2);
}

template <int KROW, int MODE, int QT>
__device__ __forceinline__ void sweep_dense_epilogue(const float* __restrict__ lds_acc,
                                                     const int32_t* __restrict__ piece_target,
                                                     const SweepFusedArgs& fa, int wave, int lane) {
  constexpr int kRow = KROW;
  const int r = lane & 31, h = lane >> 5;
  const int rt = wave & 1;
  const int nct = (fa.f_out + 31) >> 5;
  // rows of the output this lane holds in a 32 x 32 accumulator tile: 8 * (v / 4) + 4 * h + v % 4
  int32_t tg[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int tr = rt * 32 + (v >> 2) * 8 + h * 4 + (v & 3);
    tg[v] = piece_target[((int64_t)blockIdx.x * 4 + (tr >> 4)) * kSweepSlots + (tr & 15)];
  }
  const float* __restrict__ trow = lds_acc + (size_t)(rt * 32 + r) * kRow;
  // this wavefront's column tiles: ct_first, ct_first + 2, ..  (at most 4 of the at most 8).  k runs
  // in the outer loop so that a row piece of T is read from LDS once for the tiles of a pass, and the
  // operands of W for the next k group are requested before the matrix instructions of this one;
  // QT of them per pass over k (the accumulators of a pass live in registers: 16 per tile).
  const int ct_first = wave >> 1;
  const int nmine = nct > ct_first ? (nct - ct_first + 1) >> 1 : 0;
#pragma unroll 1
  for (int q0 = 0; q0 < nmine; q0 += QT) {
    const int ct0 = ct_first + 2 * q0;
    const int nmy = nmine - q0 < QT ? nmine - q0 : QT;
    sweep_floatx16 z[QT];
#pragma unroll
    for (int q = 0; q < QT; ++q)
#pragma unroll
      for (int v = 0; v < 16; ++v) z[q][v] = 0.f;
    if constexpr (MODE == 2) {
      // W as packed by sweep_pack_w_kernel with three planes: term t of W at Wp + t * (kRow / 8) * NB
      const sweep_bf16x8* __restrict__ Wp = reinterpret_cast<const sweep_bf16x8*>(fa.Wp);
      const int NB = nct * 32;
      const int64_t plane = (int64_t)(kRow / 8) * NB;
      constexpr int J = kRow / 16;
      sweep_bf16x8 cur[QT][3], nxt[QT][3];
#pragma unroll
      for (int q = 0; q < QT; ++q)
        if (q < nmy) {
#pragma unroll
          for (int t = 0; t < 3; ++t) cur[q][t] = Wp[t * plane + (int64_t)h * NB + (ct0 + 2 * q) * 32 + r];
        }
#pragma unroll 1
      for (int j = 0; j < J; ++j) {
        if (j + 1 < J) {
#pragma unroll
          for (int q = 0; q < QT; ++q)
            if (q < nmy) {
#pragma unroll
              for (int t = 0; t < 3; ++t)
                nxt[q][t] = Wp[t * plane + (int64_t)(2 * (j + 1) + h) * NB + (ct0 + 2 * q) * 32 + r];
            }
        }
        const float4 x0 = *reinterpret_cast<const float4*>(trow + 16 * j + 8 * h);
        const float4 x1 = *reinterpret_cast<const float4*>(trow + 16 * j + 8 * h + 4);
        const float xs[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
        sweep_bf16x8 a1, a2, a3;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          __bf16 t1, t2, t3;
          sweep_split3(xs[i], t1, t2, t3);
          a1[i] = t1; a2[i] = t2; a3[i] = t3;
        }
#pragma unroll
        for (int q = 0; q < QT; ++q)
          if (q < nmy) {
            z[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a3, cur[q][0], z[q], 0, 0, 0);
            z[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, cur[q][2], z[q], 0, 0, 0);
            z[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, cur[q][1], z[q], 0, 0, 0);
            z[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, cur[q][0], z[q], 0, 0, 0);
            z[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, cur[q][1], z[q], 0, 0, 0);
            z[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, cur[q][0], z[q], 0, 0, 0);
          }
#pragma unroll
        for (int q = 0; q < QT; ++q)
#pragma unroll
          for (int t = 0; t < 3; ++t) cur[q][t] = nxt[q][t];
      }
    } else if constexpr (MODE == 1) {
      // W as packed by sweep_pack_w_kernel: [k / 8][NB] vectors of 8 bfloat16 (zero beyond f_out)
      const sweep_bf16x8* __restrict__ Wp = reinterpret_cast<const sweep_bf16x8*>(fa.Wp);
      const int NB = nct * 32;
      constexpr int J = kRow / 16;
      sweep_bf16x8 cur[QT], nxt[QT];
#pragma unroll
      for (int q = 0; q < QT; ++q)
        if (q < nmy) cur[q] = Wp[(int64_t)h * NB + (ct0 + 2 * q) * 32 + r];
#pragma unroll 1
      for (int j = 0; j < J; ++j) {
        if (j + 1 < J) {
#pragma unroll
          for (int q = 0; q < QT; ++q)
            if (q < nmy) nxt[q] = Wp[(int64_t)(2 * (j + 1) + h) * NB + (ct0 + 2 * q) * 32 + r];
        }
        const float4 x0 = *reinterpret_cast<const float4*>(trow + 16 * j + 8 * h);
        const float4 x1 = *reinterpret_cast<const float4*>(trow + 16 * j + 8 * h + 4);
        sweep_bf16x8 a;
        a[0] = (__bf16)x0.x; a[1] = (__bf16)x0.y; a[2] = (__bf16)x0.z; a[3] = (__bf16)x0.w;
        a[4] = (__bf16)x1.x; a[5] = (__bf16)x1.y; a[6] = (__bf16)x1.z; a[7] = (__bf16)x1.w;
#pragma unroll
        for (int q = 0; q < QT; ++q)
          if (q < nmy) z[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, cur[q], z[q], 0, 0, 0);
#pragma unroll
        for (int q = 0; q < QT; ++q) cur[q] = nxt[q];
      }
    } else {
      constexpr int J = kRow / 8;
      float cur[QT][4], nxt[QT][4];
      auto wload = [&](int j, float (&dst)[QT][4]) {
#pragma unroll
        for (int q = 0; q < QT; ++q) {
          const int col = (ct0 + 2 * q) * 32 + r;
          const bool ok = q < nmy && col < fa.f_out;
#pragma unroll
          for (int i = 0; i < 4; ++i) dst[q][i] = ok ? fa.W[(int64_t)(8 * j + 4 * h + i) * fa.f_out + col] : 0.f;
        }
      };
      wload(0, cur);
#pragma unroll 1
      for (int j = 0; j < J; ++j) {
        if (j + 1 < J) wload(j + 1, nxt);
        const float4 x = *reinterpret_cast<const float4*>(trow + 8 * j + 4 * h);
        const float xs[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int q = 0; q < QT; ++q) {
          if (q < nmy) {
#pragma unroll
            for (int i = 0; i < 4; ++i) z[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(xs[i], cur[q][i], z[q], 0, 0, 0);
          }
        }
#pragma unroll
        for (int q = 0; q < QT; ++q)
#pragma unroll
          for (int i = 0; i < 4; ++i) cur[q][i] = nxt[q][i];
      }
    }
#pragma unroll
    for (int q = 0; q < QT; ++q) {
      const int col = (ct0 + 2 * q) * 32 + r;
      if (q >= nmy || col >= fa.f_out) continue;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        if (tg[v] < 0) continue;               // unused slot, or a piece of a split row
        const float zz = z[q][v];
        if (fa.Z) fa.Z[(int64_t)tg[v] * fa.f_out + col] = zz;
        if (fa.Hout) fa.Hout[(int64_t)tg[v] * fa.f_out + col] = fa.act == SAGNN_ACT_RELU ? (zz > 0.f ? zz : 0.f) : zz;
      }
    }
  }
}

template <int FPL, int U, bool BUF, int MODE>
__global__ __launch_bounds__(256) void spmm_sweep_fused_kernel(
    const uint32_t* __restrict__ code, const float* __restrict__ vals,
    const int32_t* __restrict__ wave_base, const int32_t* __restrict__ piece_target,
    const SpmmWsHeader* __restrict__ hdr, const float* __restrict__ B, float* __restrict__ partial,
    const SweepDims d, const SweepFusedArgs fa) {
  using vec = typename Vec<FPL>::T;
  extern __shared__ __attribute__((aligned(16))) float lds_acc[];  // [4 waves][16][64*FPL]
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t loff = lane * (FPL * 4);
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int64_t w = (int64_t)blockIdx.x * 4 + wave;
  // (the launch has whole workgroups: n_waves is a multiple of 4, checked by the launcher)
  if (hdr->magic != kSpmmMagic || hdr->generation != d.generation || hdr->n_waves != d.n_waves ||
      hdr->groups != 1)
    return;
  constexpr int kRow = 64 * FPL;  // floats per accumulator row = f_in
  float* __restrict__ my = lds_acc + (size_t)wave * kSweepSlots * kRow + lane * FPL;
  for (int s = 0; s < kSweepSlots; ++s) *reinterpret_cast<vec*>(my + s * kRow) = vec(0.f);

  const int32_t base = wave_base[w];
  const int32_t len = wave_base[w + 1] - base;  // a multiple of U (padded when built)
  const uint32_t* __restrict__ cw = code + base;
  const float* __restrict__ vw = vals + base;
  const __amdgpu_buffer_rsrc_t rs = make_rsrc(B, d.b_bytes);

  vec acc = 0.f;
  for (int32_t e = 0; e < len; e += U) {
    uint32_t c[U];
    float v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      c[u] = cw[e + u];
      v[u] = vw[e + u];
    }
    vec h[U];
#pragma unroll
    for (int u = 0; u < U; ++u) h[u] = load_row<FPL, BUF>(rs, B, c[u] & kColMask, loff, d.row_bytes, d.ldb);
#pragma unroll
    for (int u = 0; u < U; ++u) asm volatile("" : "+v"(h[u]));
#pragma unroll
    for (int u = 0; u < U; ++u) {
      acc += v[u] * h[u];
      if (c[u] >> 31) {
        vec* p = reinterpret_cast<vec*>(my + ((c[u] >> kSweepColBits) & (kSweepSlots - 1)) * kRow);
        *p += acc;
        acc = 0.f;
      }
    }
  }

  // pieces of split rows to `partial`; T rows to memory if wanted
#pragma unroll 1
  for (int s = 0; s < kSweepSlots; ++s) {
    const int32_t tgt = piece_target[w * kSweepSlots + s];
    if (tgt == INT32_MIN) continue;
    const vec r = *reinterpret_cast<const vec*>(my + s * kRow);
    if (tgt >= 0) {
      if (fa.T) *reinterpret_cast<vec*>(reinterpret_cast<char*>(fa.T + (int64_t)tgt * kRow) + loff) = r;
    } else {
      const int64_t pi = -(int64_t)tgt - 1;
      *reinterpret_cast<vec*>(reinterpret_cast<char*>(partial + pi * d.f_total + d.col0) + loff) = r;
    }
  }
  __syncthreads();

  // tiles per pass: 4 at f = 256 (the LDS already limits a CU to two workgroups; 2 with three operand
  // terms per tile in registers), 1 below
  sweep_dense_epilogue<kRow, MODE, (FPL == 4 ? (MODE == 2 ? 2 : 4) : 1)>(lds_acc, piece_target, fa, wave, (int)lane);
}

// W (f_in x f_out, row-major fp32) -> [f_in / 8][NB] vectors of 8 bfloat16 (k fastest), NB = f_out
// rounded up to 32, zero beyond f_out: one 16-byte load then gives a lane its matrix-core operand
// planes = 3: the three bfloat16 terms of every element, one plane of that layout per term
__global__ __launch_bounds__(256) void sweep_pack_w_kernel(const float* __restrict__ W, int32_t f_in, int32_t f_out,
                                                           int32_t NB, __bf16* __restrict__ Wp, int32_t planes) {
  const int idx = blockIdx.x * 256 + threadIdx.x;     // one (k / 8, n) vector per thread
  if (idx >= (f_in / 8) * NB) return;
  const int kg = idx / NB, n = idx - kg * NB;
  const int64_t plane = (int64_t)(f_in / 8) * NB * 8;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float w = n < f_out ? W[(int64_t)(kg * 8 + i) * f_out + n] : 0.f;
    if (planes == 3)
      sweep_split3(w, Wp[(int64_t)idx * 8 + i], Wp[plane + (int64_t)idx * 8 + i], Wp[2 * plane + (int64_t)idx * 8 + i]);
    else
      Wp[(int64_t)idx * 8 + i] = (__bf16)w;
  }
}

// Lane-group variant: the wavefront carries R independent streams (zipped in memory), lane
// group g = lanes [g*64/R, (g+1)*64/R) walks stream g.  A group's 64/R lanes move one whole row
// of B with V floats (16 bytes at V = 4) per lane, so one load instruction serves R entries.
// Column ids and values still arrive by scalar loads; a lane picks its group's pair with
// selects (the row offset is multiplied on the scalar side first).  Flushes are per group:
// lanes of other groups are masked off by the divergent branch.
// FUSE: 0 the product alone; 1 / 2 / 3 the layer form: the kernel ends with the dense transform of the
// workgroup's rows (fp32 / bfloat16 / three-term operands, see sweep_dense_epilogue) instead of storing T (C is
// then only written if the caller wants T as a by-product: fa.T).
template <int V, int R, int U, bool BUF, int FUSE = 0>
__global__ __launch_bounds__(256) void spmm_sweep_group_kernel(
    const uint32_t* __restrict__ code, const float* __restrict__ vals,
    const int32_t* __restrict__ wave_base, const int32_t* __restrict__ piece_target,
    const SpmmWsHeader* __restrict__ hdr, const float* __restrict__ B, float* __restrict__ C,
    float* __restrict__ partial, const int32_t* __restrict__ sync_off,
    uint32_t* __restrict__ barrier, const float* __restrict__ sched, const SweepDims d,
    const SweepFusedArgs fa) {
  using vec = typename Vec<V>::T;
  constexpr int LG = 64 / R;             // lanes per group = lanes per row
  constexpr int kRow = LG * V;           // floats per row of this launch
  extern __shared__ __attribute__((aligned(16))) float lds_acc[];  // [4 waves][d.slots][kRow]
  const int SL = d.slots / R;            // slots per group
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t gid = lane / LG, lig = lane % LG;
  const uint32_t loff = lig * (V * 4);
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int64_t w = (int64_t)blockIdx.x * 4 + wave;
  if (w >= d.n_waves) return;
  if (hdr->magic != kSpmmMagic || hdr->generation != d.generation || hdr->n_waves != d.n_waves ||
      hdr->groups != R)
    return;
  float* __restrict__ my = lds_acc + (size_t)wave * d.slots * kRow + lig * V;
  for (int ls = 0; ls < SL; ++ls) *reinterpret_cast<vec*>(my + (gid * SL + ls) * kRow) = vec(0.f);

  const int32_t base = wave_base[w];
  const int32_t steps = (wave_base[w + 1] - base) / R;   // a multiple of U (padded when built)
  const uint32_t* __restrict__ cw = code + base;
  const float* __restrict__ vw = vals + base;
  const __amdgpu_buffer_rsrc_t rs = make_rsrc(B, d.b_bytes);
  // interval boundaries of this wavefront's stream (whole batches) and the barrier it shares
  // with the workgroups of its cohort on its XCD
  const bool with_barrier = d.n_intervals > 1;     // negative: same layout, no barriers
  const int n_iv = d.n_intervals < 0 ? -d.n_intervals : d.n_intervals;
  const int32_t* __restrict__ so = sync_off + w * (kSweepMaxIntervals + 1);
  uint32_t expected = 0;
  int bar_slot0 = 0;
  if (with_barrier) {
    const int64_t cohort = (int64_t)blockIdx.x / d.wg_per_cohort;
    const int64_t first = cohort * d.wg_per_cohort;
    int64_t last = first + d.wg_per_cohort;
    if (last > (int64_t)gridDim.x) last = gridDim.x;
    const int xg = (int)(blockIdx.x & 7);
    // workgroups b in [first, last) with b mod 8 == xg (first is a multiple of 8)
    expected = (uint32_t)((last - first - xg + 7) / 8) + (uint32_t)d.sync_test_extra;
    bar_slot0 = (int)((cohort * 8 + xg) * n_iv);
  }

  const bool paced = d.pace_ticks > 0.f && n_iv > 1;
  const uint64_t t_start = paced ? wall_clock64() : 0ull;

  vec acc = 0.f;
  int32_t e = 0;
  for (int iv = 0; iv < n_iv; ++iv) {
    const int32_t e_end = iv + 1 < n_iv ? so[iv + 1] : steps;
    for (; e < e_end; e += U) {
      uint32_t c[U][R];
      float v[U][R];
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int g = 0; g < R; ++g) {
          c[u][g] = cw[(e + u) * R + g];
          v[u][g] = vw[(e + u) * R + g];
        }
      uint32_t mc[U];
      float mv[U];
      vec h[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        mc[u] = c[u][0];
        mv[u] = v[u][0];
        if constexpr (BUF) {
          uint32_t off = (c[u][0] & kColMask) * d.row_bytes;
#pragma unroll
          for (int g = 1; g < R; ++g)
            if (gid == (uint32_t)g) {
              mc[u] = c[u][g];
              mv[u] = v[u][g];
              off = (c[u][g] & kColMask) * d.row_bytes;
            }
          off += loff;
          if constexpr (V == 1) h[u] = __builtin_bit_cast(vec, __builtin_amdgcn_raw_buffer_load_b32(rs, off, 0, 0));
          else if constexpr (V == 2) h[u] = __builtin_bit_cast(vec, __builtin_amdgcn_raw_buffer_load_b64(rs, off, 0, 0));
          else h[u] = __builtin_bit_cast(vec, __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0));
        } else {
          const char* rowp = reinterpret_cast<const char*>(B + (int64_t)(c[u][0] & kColMask) * d.ldb);
#pragma unroll
          for (int g = 1; g < R; ++g)
            if (gid == (uint32_t)g) {
              mc[u] = c[u][g];
              mv[u] = v[u][g];
              rowp = reinterpret_cast<const char*>(B + (int64_t)(c[u][g] & kColMask) * d.ldb);
            }
          h[u] = *reinterpret_cast<const vec*>(rowp + loff);
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) asm volatile("" : "+v"(h[u]));
#pragma unroll
      for (int u = 0; u < U; ++u) {
        acc += mv[u] * h[u];
        if (mc[u] >> 31) {   // last entry of a (piece, slab) segment of this lane's group
          vec* p = reinterpret_cast<vec*>(my + ((mc[u] >> kSweepColBits) & (kSweepSlots - 1)) * kRow);
          *p += acc;
          acc = 0.f;
        }
      }
    }
    // between two intervals: wait for the cohort (barrier mode) or hold the wavefront to the
    // schedule (pacing); a wavefront with nothing in an interval still takes part
    if (iv + 1 < n_iv) {
      if (with_barrier) sweep_interval_barrier(barrier, bar_slot0 + iv, expected, d.sync_timeout_ticks);
      else if (paced) sweep_pace_until(t_start, d.pace_ticks * sched[iv + 1]);
    }
  }

#pragma unroll 1
  for (int ls = 0; ls < SL; ++ls) {
    const int slot = (int)gid * SL + ls;
    const int32_t tgt = piece_target[w * kSweepSlots + slot];
    if (tgt == INT32_MIN) continue;
    vec r = *reinterpret_cast<const vec*>(my + slot * kRow);
    if (tgt >= 0) {
      if constexpr (FUSE != 0) {
        if (fa.T) *reinterpret_cast<vec*>(reinterpret_cast<char*>(fa.T + (int64_t)tgt * kRow) + loff) = r;
      } else {
        vec* p = reinterpret_cast<vec*>(reinterpret_cast<char*>(C + (int64_t)tgt * d.ldc) + loff);
        if (d.accumulate) r += *p;
        *p = r;
      }
    } else {
      const int64_t pi = -(int64_t)tgt - 1;
      *reinterpret_cast<vec*>(reinterpret_cast<char*>(partial + pi * d.f_total + d.col0) + loff) = r;
    }
  }
  if constexpr (FUSE != 0) {
    // (whole workgroups: the launcher only takes this form when n_waves is a multiple of 4 and
    // every wavefront owns 16 slots)
    __syncthreads();
    sweep_dense_epilogue<kRow, FUSE - 1, 1>(lds_acc, piece_target, fa, wave, (int)lane);
  }
}

// Narrow operands (rows of 64 / 128 bytes): R = 16 / 8 lane groups of 4 / 8 lanes.  Too many
// groups for scalar selects, so a batch of 64 stream words (64/R steps x R groups) is fetched with
// one coalesced load per array and a step's group takes its word with a lane permute.  With 16
// groups each group owns a single piece and its register accumulator is the piece's accumulator
// (no LDS at all); with 8 groups two pieces per group share it through LDS as in the wide kernels.
template <int R, bool BUF>
__global__ __launch_bounds__(256) void spmm_sweep_perm_kernel(
    const uint32_t* __restrict__ code, const float* __restrict__ vals,
    const int32_t* __restrict__ wave_base, const int32_t* __restrict__ piece_target,
    const SpmmWsHeader* __restrict__ hdr, const float* __restrict__ B, float* __restrict__ C,
    float* __restrict__ partial, const SweepDims d) {
  typedef float vec __attribute__((ext_vector_type(4)));
  constexpr int LG = 64 / R;             // lanes per group = lanes per row
  constexpr int kRow = LG * 4;           // floats per row
  constexpr int SL = kSweepSlots / R;    // pieces per group
  constexpr int UB = 64 / R;             // steps per batch of 64 stream words
  constexpr int NB = 8 / UB;             // batches per iteration: 8 steps (gathers) in flight
  extern __shared__ __attribute__((aligned(16))) float lds_acc[];  // [4 waves][16 slots][kRow], SL > 1 only
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t gid = lane / LG, lig = lane % LG;
  const uint32_t loff = lig * 16;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int64_t w = (int64_t)blockIdx.x * 4 + wave;
  if (w >= d.n_waves) return;
  if (hdr->magic != kSpmmMagic || hdr->generation != d.generation || hdr->n_waves != d.n_waves ||
      hdr->groups != R)
    return;
  float* __restrict__ my = lds_acc + (size_t)wave * kSweepSlots * kRow + lig * 4;
  if constexpr (SL > 1) {
#pragma unroll
    for (int ls = 0; ls < SL; ++ls) *reinterpret_cast<vec*>(my + (gid * SL + ls) * kRow) = vec(0.f);
  }
  const int32_t base = wave_base[w];
  const int32_t steps = (wave_base[w + 1] - base) / R;   // a multiple of 8 (padded when built)
  const uint32_t* __restrict__ cw = code + base;
  const float* __restrict__ vw = vals + base;
  const __amdgpu_buffer_rsrc_t rs = make_rsrc(B, d.b_bytes);

  vec acc = 0.f, tot = 0.f;
  uint32_t cb[NB];
  float vb[NB];
#pragma unroll
  for (int q = 0; q < NB; ++q) {
    cb[q] = steps > 0 ? cw[q * 64 + lane] : 0u;
    vb[q] = steps > 0 ? vw[q * 64 + lane] : 0.f;
  }
  for (int32_t e = 0; e < steps; e += 8) {
    // the next iteration's stream words are requested before this one's gathers are waited for
    const bool more = e + 8 < steps;
    uint32_t ncb[NB];
    float nvb[NB];
#pragma unroll
    for (int q = 0; q < NB; ++q) {
      ncb[q] = more ? cw[(e + 8) * R + q * 64 + lane] : 0u;
      nvb[q] = more ? vw[(e + 8) * R + q * 64 + lane] : 0.f;
    }
    uint32_t mc[8];
    float mv[8];
    vec h[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      mc[u] = (uint32_t)__shfl((int)cb[u / UB], (u % UB) * R + (int)gid, 64);
      mv[u] = __shfl(vb[u / UB], (u % UB) * R + (int)gid, 64);
      const uint32_t col = mc[u] & kColMask;
      if constexpr (BUF) {
        h[u] = __builtin_bit_cast(vec, __builtin_amdgcn_raw_buffer_load_b128(rs, col * d.row_bytes + loff, 0, 0));
      } else {
        h[u] = *reinterpret_cast<const vec*>(reinterpret_cast<const char*>(B + (int64_t)col * d.ldb) + loff);
      }
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) asm volatile("" : "+v"(h[u]));
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      acc += mv[u] * h[u];
      if constexpr (SL > 1) {
        if (mc[u] >> 31) {   // last entry of a (piece, slab) segment of this lane's group
          vec* p = reinterpret_cast<vec*>(my + ((mc[u] >> kSweepColBits) & (kSweepSlots - 1)) * kRow);
          *p += acc;
          acc = 0.f;
        }
      }
    }
    if constexpr (SL == 1) {
      // no slots to flush into: fold the running sum every 64 entries instead (two-level sum)
      if ((e & 63) == 56) {
        tot += acc;
        acc = 0.f;
      }
    }
#pragma unroll
    for (int q = 0; q < NB; ++q) {
      cb[q] = ncb[q];
      vb[q] = nvb[q];
    }
  }
  if constexpr (SL == 1) acc += tot;

#pragma unroll 1
  for (int ls = 0; ls < SL; ++ls) {
    const int slot = (int)gid * SL + ls;
    const int32_t tgt = piece_target[w * kSweepSlots + slot];
    if (tgt == INT32_MIN) continue;
    vec r = acc;
    if constexpr (SL > 1) r = *reinterpret_cast<const vec*>(my + slot * kRow);
    if (tgt >= 0) {
      vec* p = reinterpret_cast<vec*>(reinterpret_cast<char*>(C + (int64_t)tgt * d.ldc) + loff);
      if (d.accumulate) r += *p;
      *p = r;
    } else {
      const int64_t pi = -(int64_t)tgt - 1;
      *reinterpret_cast<vec*>(reinterpret_cast<char*>(partial + pi * d.f_total + d.col0) + loff) = r;
    }
  }
}

// rows cut into several pieces: C[row] (+)= sum of the pieces' partial rows, fixed order
__global__ __launch_bounds__(256) void sweep_combine_kernel(
    const int32_t* __restrict__ multi_row, const int32_t* __restrict__ multi_first,
    const float* __restrict__ partial, const SpmmWsHeader* __restrict__ hdr, uint64_t generation,
    int64_t n_multi, float* __restrict__ C, int64_t ldc, int32_t f_total, int32_t accumulate) {
  const int lane = threadIdx.x & 63;
  const int64_t q = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6;
  if (q >= n_multi) return;
  if (hdr->magic != kSpmmMagic || hdr->generation != generation) return;
  const int32_t row = multi_row[q];
  const int32_t a = multi_first[q], b = multi_first[q + 1];
  for (int c4 = lane; c4 * 4 < f_total; c4 += 64) {
    float4 s0 = make_float4(0.f, 0.f, 0.f, 0.f), s1 = s0;
    int32_t j = a;
    for (; j + 2 <= b; j += 2) {
      const float4 t0 = *reinterpret_cast<const float4*>(partial + (int64_t)j * f_total + c4 * 4);
      const float4 t1 = *reinterpret_cast<const float4*>(partial + (int64_t)(j + 1) * f_total + c4 * 4);
      s0.x += t0.x; s0.y += t0.y; s0.z += t0.z; s0.w += t0.w;
      s1.x += t1.x; s1.y += t1.y; s1.z += t1.z; s1.w += t1.w;
    }
    if (j < b) {
      const float4 t0 = *reinterpret_cast<const float4*>(partial + (int64_t)j * f_total + c4 * 4);
      s0.x += t0.x; s0.y += t0.y; s0.z += t0.z; s0.w += t0.w;
    }
    float4* p = reinterpret_cast<float4*>(C + (int64_t)row * ldc + c4 * 4);
    float4 o = accumulate ? *p : make_float4(0.f, 0.f, 0.f, 0.f);
    o.x += s0.x + s1.x; o.y += s0.y + s1.y; o.z += s0.z + s1.z; o.w += s0.w + s1.w;
    *p = o;
  }
}

std::atomic<uint64_t> g_generation{1};

}  // namespace

// ---------------------------------------------------------------------------------------
// host side of the preparation: the launch shape (lane groups, slots, windows, wavefronts per
// window) is decided here from a handful of totals; classifying rows, cutting long rows into
// pieces, dealing the pieces to the streams of the wavefronts (largest first, each to the
// shortest stream so far, so the streams have nearly equal lengths) and the compacted short-row
// CSR are device work (sweep_plan.hip), as is the layout of the streams (the passes above).
int sweep_prepare(const int32_t* d_rowptr, const int32_t* d_colidx, const float* d_val, int64_t m,
                  int64_t k, int64_t nnz, int32_t f, char* ws, const SpmmWsLayout& L,
                  const sagnn_spmm_options& opt, hipStream_t s, SweepPlanResult* out) {
  out->use_sweep = false;
  const int force = opt.schedule == 1 ? 0 : (opt.schedule == 2 ? 1 : -1);
  if (force == 0 || nnz < 4096 || k <= 0 || k >= (1ll << kSweepColBits) || m <= 0) return SAGNN_OK;
  const int64_t b_bytes = k * (int64_t)f * 4;
  // worth it only if B is much larger than an L2 (the long-row share is checked below)
  if (force != 1 && (nnz < (1 << 20) || b_bytes <= (8ll << 20))) return SAGNN_OK;

  if (!sweep_plan_fits(L)) return SAGNN_OK;
  int piece_max = opt.piece > 0 ? opt.piece : 4096;
  if (piece_max < 1024) piece_max = 1024;
  if (piece_max > 32768) piece_max = 32768;
  const int64_t slab_bytes = opt.slab_kb < 0 ? 0 : (int64_t)(opt.slab_kb > 0 ? opt.slab_kb : 4096) << 10;
  int64_t S = slab_bytes >= (1 << 16) ? 8 * ceil_div(b_bytes, 8 * slab_bytes) : kSweepMaxSlabs;
  if (S < 8) S = 8;
  if (S > kSweepMaxSlabs) S = kSweepMaxSlabs;
  const int64_t width = ceil_div(k, S);

  // Row classification, the short-row CSR, the list of split rows and one record per piece are
  // made on the device (the long-row threshold is chosen there from the degree distribution);
  // the host gets the totals.
  SweepRowTotals tot{};
  {
    const int rc = sweep_plan_rows(d_rowptr, m, nnz, opt.min_long, piece_max, ws, L, s, &tot, opt.short_rows >= 0);
    if (rc != SAGNN_OK) return rc;
  }
  if (tot.bad) return SAGNN_OK;   // not a CSR row pointer for this nnz: keep the plain schedule
  const int64_t P = tot.pieces, short_rows = tot.short_rows, short_entries = tot.short_entries;
  const int64_t long_entries = nnz - short_entries;
  const bool has_empty = tot.has_empty;

  // Lane groups: at f = 128 half a wavefront, at f = 64 a quarter, moves a whole row of B with
  // 16 bytes per lane, so one load instruction serves 2 / 4 entries (the vector-memory issue
  // rate, not bandwidth, bounds B-in-cache cases).  Other widths keep one row per instruction.
  // They pay when the rows of B are re-used from cache (issue-bound: 233 k-vertex graph
  // 3.38 -> 2.63 ms, 2.45 M-vertex graph 4.85 -> 4.62 ms) and cost ~3 % when almost every gather
  // misses (rank share of the 111 M-vertex graph, 2.6 entries per row of B): decided below by
  // the average number of swept entries per row of B.
  // Narrow operands (f = 32, 16: rows of 128 / 64 bytes, 8 / 4 lanes each) exist only in the
  // grouped form, 8 / 16 rows per load.
  // Wider operands (multiples of 64 above 128) can be taken as 128-wide slabs by the two-group
  // kernels (a last slab of 64 is served by the same streams): an option, see sagnn_spmm_options.
  const bool narrow_slabs = opt.slab_width == 128 && f > 128 && (f & 63) == 0 && opt.groups != 1;
  int64_t R = (f == 128 || narrow_slabs) ? 2 : (f == 64 ? 4 : (f == 32 ? 8 : (f == 16 ? 16 : 1)));
  if (opt.groups == 1 && f >= 64) R = 1;
  if (force != 1 && long_entries * 10 < nnz * 3) return SAGNN_OK;   // < 30 % of the entries
  if (opt.groups != 2 && long_entries < 8 * k) {
    if (f < 64) return SAGNN_OK;   // no one-row-per-instruction form below 64: plain schedule
    R = 1;
  }
  if (P <= 0 || P > L.max_pieces) return SAGNN_OK;
  if (tot.multi_rows > L.max_multi_rows || tot.multi_pieces > L.max_multi_pieces) return SAGNN_OK;

  // Accumulator rows per wavefront.  A launch of width 128 with 16 rows per wavefront needs
  // 32768 bytes of LDS per workgroup, of which a CU holds four, not five (measured; the LDS
  // is handed out in units that make 5 x 32768 overshoot 160 KB).  14 rows (lane groups, 7 each)
  // or 15 rows bring the fifth workgroup in, 20 wavefronts and 280 / 300 rows per CU instead
  // of 16 and 256 -- measured slower free-running on the 2.45 M-vertex graph (5.4 against
  // 4.5 ms: more wavefronts drift apart more) and equal under pacing, so it is an option only.
  const bool has_128_slab = narrow_slabs || (f % 256) == 128 || (f % 256) == 192;
  const int64_t slots = has_128_slab && opt.narrow_slots == 1 ? (R == 2 ? 14 : 15) : kSweepSlots;
  // Pieces per wavefront: all slots when there are plenty of pieces; fewer when that would
  // leave the chip short of wavefronts (a row block of a partitioned graph has few long rows).
  int64_t slots_used = ceil_div(P, (int64_t)(opt.min_waves > 0 ? opt.min_waves : 8192));
  if (slots_used < R) slots_used = R;          // every lane group of a wavefront gets a piece
  if (slots_used > slots) slots_used = slots;
  if (ceil_div(P, slots_used) + 64 > L.max_waves - 8) slots_used = slots;
  // Pieces are dealt window by window.  A window is a run of consecutive long rows holding a
  // few times as many pieces as the chip keeps resident at once (LDS-limited); inside a window
  // the pieces are sorted by size and dealt longest-first, so its wavefronts have nearly equal
  // stream lengths (they pass the slabs in step).  A matrix of up to ~4 generations is one
  // window (measured best on randomly labelled graphs: 4.95 ms against 5.4 ms with one window
  // per generation on the 2.45 M-vertex R-MAT graph); a larger one whose row order carries
  // locality (a partitioned graph) keeps it, because a window only touches the part of B its
  // rows' neighbourhoods live in (2 M-vertex community-ordered graph: 13.9 -> 11.4 ms).
  const int64_t fw_max = narrow_slabs ? 128 : (f >= 256 ? 256 : (f >= 128 ? 128 : f));   // widest launch of a call
  int64_t wg_per_cu = lds_resident_workgroups((size_t)(4ll * slots * fw_max * 4));
  if (wg_per_cu < 1) wg_per_cu = 1;
  int n_cus = 256;
  {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      n_cus = v;
  }
  const int64_t resident_waves = (int64_t)n_cus * wg_per_cu * 4;
  int64_t window = resident_waves * slots_used;              // pieces per window
  {
    const int pct = opt.window_pct < 0 ? 0 : (opt.window_pct > 0 ? opt.window_pct : 400);
    window = pct <= 0 ? P : std::max<int64_t>(slots_used, window * pct / 100);
  }
  if (window > P) window = P;
  if (ceil_div(P, window) > kSweepMaxWindows) window = ceil_div(P, kSweepMaxWindows);
  const int64_t nwin = ceil_div(P, window);
  // Wavefronts in all: whole generations of resident wavefronts when there is more than one
  // (the last generation then runs at the same occupancy, and under pacing at the same speed, as
  // the others), else as few as the slots allow.
  int64_t n_target_waves = ceil_div(P, slots_used);
  if (n_target_waves > resident_waves) {
    const int64_t up = round_up((size_t)n_target_waves, (size_t)resident_waves);
    if (up + 64 <= L.max_waves - 8) n_target_waves = up;
  }
  std::vector<int64_t> win_entries(1, long_entries);
  if (nwin > 1) {
    const int rc = sweep_plan_window_entries(ws, L, P, window, (int32_t)nwin, s, &win_entries);
    if (rc != SAGNN_OK) return rc;
  }
  // wavefronts of a window: as many as keep the stream length equal to the global average (equal
  // lengths in ALL windows keep successive generations in step), but never fewer than the slots
  // allow.  With R lane groups a wavefront carries R independent streams (group g owns slots
  // g*SL ..); the unit of dealing is then the group stream.
  const int64_t SL = slots / R;                 // slots per group stream
  std::vector<int32_t> win_unit0((size_t)nwin + 1);   // first stream of every window
  int64_t NW = 0;
  for (int64_t w = 0; w < nwin; ++w) {
    const int64_t a = w * window, b = std::min(P, a + window);
    const double target_len = (double)long_entries / (double)n_target_waves;
    int64_t nw = (int64_t)((double)win_entries[(size_t)w] / target_len + 0.5);
    nw = std::max(nw, ceil_div(b - a, slots));
    nw = std::max<int64_t>(nw, 1);
    nw = std::min(nw, b - a);
    win_unit0[(size_t)w] = (int32_t)(NW * R);
    NW += nw;
  }
  win_unit0[(size_t)nwin] = (int32_t)(NW * R);
  // whole workgroups of four wavefronts (the last ones may own no piece): the kernels' workgroup
  // barriers then never meet a wavefront that has left
  const int64_t NW4 = (NW + 3) / 4 * 4;
  if (NW4 > L.max_waves - 1) return SAGNN_OK;   // cannot happen with the bounds above; plain schedule
  // Option: the short rows are swept too, as whole rows -- 16 per wavefront, behind the wavefronts
  // of the long rows, every row one segment of its wavefront's stream -- instead of going through
  // the nonzero-splitting kernel.  Every row then ends in a wavefront's accumulator rows, which is
  // what the layer form with the dense transform as the sweep's epilogue needs.
  // Measured never slower than the nonzero-splitting kernel on the power-law graphs (233 k vertices:
  // 2.54 -> 2.50 ms, 2.45 M vertices: 2.78 -> 2.62 ms at f = 64, 4.24 -> 4.19 ms at f = 128), also
  // when the short rows are very short (2 M rows of which 92 % hold one entry each: 3.50 -> 3.38 ms).
  bool whole_rows = opt.short_rows >= 0 &&
                    short_rows > 0 && tot.min_long <= 255 && slots == kSweepSlots && R <= 4 &&
                    P + short_rows <= L.max_pieces && opt.sync_slabs <= 0 && opt.barriers != 1 &&
                    opt.pace_ps_per_step <= 0;
  int64_t NWT4 = NW4;
  if (whole_rows) {
    NWT4 = NW4 + (ceil_div(short_rows, (int64_t)kSweepSlots) + 3) / 4 * 4;
    if (NWT4 > L.max_waves - 1) {
      whole_rows = false;
      NWT4 = NW4;
    }
  }
  const int64_t first_whole_row_wave = whole_rows ? NW4 : INT64_MAX;
  const int64_t short_entries_csr = whole_rows ? 0 : short_entries;   // entries of the compacted short-row CSR
  // Inside a window: largest piece first, each to the stream that is shortest so far and still
  // has a free slot.  Streams come out equal to within a piece of the smallest size class, which
  // keeps the wavefronts in step from slab to slab.
  {
    const bool snake = R == 1 && opt.snake == 1;
    int rc = sweep_plan_deal(ws, L, P, window, win_unit0.data(), (int32_t)nwin, NWT4, (int32_t)R,
                             (int32_t)SL, snake, s);
    if (rc != SAGNN_OK) return rc;
    if (whole_rows) {
      rc = sweep_plan_deal_short(ws, L, P, short_rows, NW4, s);
      if (rc != SAGNN_OK) return rc;
    }
  }

  // Interval barriers (lane-group kernels only): every `sync_slabs` slabs the workgroups of an
  // XCD that run together wait for each other.  Decided here, laid out by the device passes.
  // (the interval layout costs ~3 % of padding, so it is only made when something will use it)
  int64_t sync_slabs = opt.sync_slabs < 0 ? 0 : (opt.sync_slabs > 0 ? opt.sync_slabs : 16);
  if (opt.barriers != 1 && opt.pace_ps_per_step <= 0 && opt.sync_slabs <= 0) sync_slabs = 0;
  if ((R != 2 && R != 4) || whole_rows) sync_slabs = 0;   // (whole-row wavefronts have no slab intervals)
  if (sync_slabs > 0 && ceil_div(S, sync_slabs) > kSweepMaxIntervals) sync_slabs = ceil_div(S, kSweepMaxIntervals);
  int64_t NI = sync_slabs > 0 ? ceil_div(S, sync_slabs) : 1;
  if (NI <= 1) { NI = 1; sync_slabs = 0; }

  // long rows must be column-sorted for the slab segmentation
  int32_t* d_flag = reinterpret_cast<int32_t*>(ws + L.carry);  // scratch until the first product; zeroed by the row pass
  hipLaunchKernelGGL(sweep_check_sorted_kernel, dim3((unsigned)ceil_div(NW4 * kSweepSlots, 4)), dim3(256),
                     0, s, d_rowptr, d_colidx, reinterpret_cast<const int32_t*>(ws + L.piece_info),
                     NW4 * kSweepSlots, (uint32_t)(k - 1), d_flag);
  SAGNN_LAUNCH_CHECK();

  const uint32_t kmax = (uint32_t)(k - 1);
  const int32_t* d_info = reinterpret_cast<const int32_t*>(ws + L.piece_info);
  int32_t* d_wave_base = reinterpret_cast<int32_t*>(ws + L.wave_base);
  int32_t* d_wave_steps = reinterpret_cast<int32_t*>(ws + L.wave_steps);
  int32_t* d_sync_off = reinterpret_cast<int32_t*>(ws + L.sync_off);
  const size_t count_lds = sweep_count_lds_bytes(S), build_lds = sweep_build_lds_bytes(S);
  SAGNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(sweep_count_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)count_lds));
  SAGNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(sweep_build_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)build_lds));
  int64_t stream_len = 0, short_base = 0;
  for (int attempt = 0; attempt < 2; ++attempt) {
    hipLaunchKernelGGL(sweep_count_kernel, dim3((unsigned)NWT4), dim3(kBuildThreads), count_lds, s, d_rowptr,
                       d_colidx, d_info, (int32_t)S, (int32_t)width, kmax, (int32_t)R, (int32_t)SL, (int32_t)NI,
                       (int32_t)sync_slabs, d_sync_off, d_wave_steps, first_whole_row_wave);
    SAGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(sweep_scan_kernel, dim3(1), dim3(1024), 0, s, d_wave_steps, NWT4, (int32_t)R,
                       d_wave_base, d_flag + 1);
    SAGNN_LAUNCH_CHECK();
    int32_t h_flags[4] = {0, 0, 0, 0}, h_total = 0;
    SAGNN_HIP(hipMemcpyAsync(h_flags, d_flag, 16, hipMemcpyDeviceToHost, s));
    SAGNN_HIP(hipMemcpyAsync(&h_total, d_wave_base + NWT4, 4, hipMemcpyDeviceToHost, s));
    SAGNN_HIP(hipStreamSynchronize(s));    // also: win_unit0 has been consumed
    if (h_flags[0] || h_flags[2]) return SAGNN_OK;   // unsorted long row, column out of range, pieces left over: plain schedule
    stream_len = h_total;
    short_base = (int64_t)round_up((size_t)stream_len + 64, 256);
    const bool fits = !h_flags[1] && short_base + short_entries_csr + kSpmmChunk <= L.stream_cap;
    if (fits) break;
    if (attempt == 1 || NI == 1) return SAGNN_OK;
    NI = 1;                                // the interval padding did not fit: lay out without it
    sync_slabs = 0;
  }

  hipLaunchKernelGGL(sweep_sched_kernel, dim3((unsigned)(NI + 2)), dim3(256), 0, s, d_sync_off, NWT4, (int32_t)NI,
                     reinterpret_cast<float*>(ws + L.sched));
  SAGNN_LAUNCH_CHECK();
  float steps[2] = {0.f, 0.f};   // mean, max over the wavefronts
  SAGNN_HIP(hipMemcpyAsync(steps, reinterpret_cast<float*>(ws + L.sched) + NI, 8, hipMemcpyDeviceToHost, s));
  hipLaunchKernelGGL(sweep_build_kernel, dim3((unsigned)NWT4), dim3(kBuildThreads), build_lds, s, d_rowptr,
                     d_colidx, d_val, d_info, d_wave_base, d_sync_off, (int32_t)S, (int32_t)width, kmax,
                     (int32_t)R, (int32_t)SL, (int32_t)NI, (int32_t)sync_slabs, reinterpret_cast<uint32_t*>(ws + L.code),
                     reinterpret_cast<float*>(ws + L.vals), first_whole_row_wave);
  SAGNN_LAUNCH_CHECK();
  // zero the gap between the long stream and the short entries (tail batches read into it)
  hipLaunchKernelGGL(sweep_zero_gap_kernel, dim3(1), dim3(256), 0, s,
                     reinterpret_cast<uint32_t*>(ws + L.code) + stream_len,
                     reinterpret_cast<float*>(ws + L.vals) + stream_len, (int32_t)(short_base - stream_len));
  SAGNN_LAUNCH_CHECK();
  if (short_rows > 0 && !whole_rows) {
    hipLaunchKernelGGL(sweep_short_copy_kernel, dim3((unsigned)ceil_div(short_rows, 256)), dim3(256), 0, s,
                       d_rowptr, d_colidx, d_val, reinterpret_cast<const int32_t*>(ws + L.rowptr_s),
                       reinterpret_cast<const int32_t*>(ws + L.rowmap_s), short_rows,
                       reinterpret_cast<int32_t*>(ws + L.code) + short_base,
                       reinterpret_cast<float*>(ws + L.vals) + short_base);
    SAGNN_LAUNCH_CHECK();
  }

  SpmmWsHeader& h = out->hdr;
  h = SpmmWsHeader{};
  h.magic = kSpmmMagic;
  h.has_empty_rows = has_empty ? 1 : 0;
  h.m = m; h.nnz = nnz; h.f = f; h.mode = 1;
  h.generation = g_generation.fetch_add(1);
  h.c_rows = whole_rows ? 0 : short_rows; h.c_nnz = short_entries_csr; h.c_nchunks = spmm_nchunks(short_entries_csr);
  h.n_waves = NWT4; h.n_long_entries = stream_len;   // padded length of the sweep streams
  h.n_multi_rows = tot.multi_rows; h.n_multi_pieces = tot.multi_pieces;
  h.n_slabs = (int32_t)S; h.slab_width = (int32_t)width;
  h.groups = (int32_t)R;
  h.n_intervals = (int32_t)NI; h.sync_slabs = (int32_t)sync_slabs;
  h.sync_timeout_ticks = (opt.sync_timeout_us > 0 ? opt.sync_timeout_us : 200) * 100;
  h.sync_test_extra = opt.sync_test_extra > 0 ? opt.sync_test_extra : 0;
  h.slots = (int32_t)slots;
  h.barriers = opt.barriers == 1 && sync_slabs > 0 ? 1 : 0;
  h.pace_ps_per_step = sync_slabs > 0 && !h.barriers ? opt.pace_ps_per_step : 0;
  h.max_slab = narrow_slabs && R == 2 ? 128 : 256;
  SAGNN_HIP(hipStreamSynchronize(s));     // the step counts have arrived
  out->mean_steps = steps[0];
  out->max_steps = steps[1];
  out->use_sweep = true;
  return SAGNN_OK;
}

uint64_t spmm_next_generation() { return g_generation.fetch_add(1); }

namespace {
// workgroups of a kernel that are resident at once on the whole device, for the cohort size of
// the interval barriers: CUs x workgroups per CU as the runtime reports them for this kernel
// and its LDS size, rounded down to a multiple of 8 (one share per XCD).  0 if unknown.
int resident_workgroups(const void* kern, size_t lds) {
  int dev = 0, cus = 0, per_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, 256, lds) != hipSuccess) return 0;
  // the runtime's figure is too high where the LDS is what limits (see lds_resident_workgroups):
  // assuming too few resident workgroups only makes a cohort smaller, assuming too many would
  // make every barrier run into its time limit
  const int by_lds = lds_resident_workgroups(lds);
  if (per_cu > by_lds) per_cu = by_lds;
  const int64_t n = (int64_t)cus * per_cu / 8 * 8;
  return n > 0 && n < (1 << 30) ? (int)n : 0;
}
}  // namespace

namespace {
// lane-group kernels: fuse = 0 product, 1 / 2 / 3 layer form with fp32 / bfloat16 / three-term operands
template <int V, int R, bool BUF>
auto group_kernel_of(int fuse) {
  if (fuse == 1) return &spmm_sweep_group_kernel<V, R, 8, BUF, 1>;
  if (fuse == 2) return &spmm_sweep_group_kernel<V, R, 8, BUF, 2>;
  if (fuse == 3) return &spmm_sweep_group_kernel<V, R, 8, BUF, 3>;
  return &spmm_sweep_group_kernel<V, R, 8, BUF, 0>;
}
}  // namespace

int sweep_launch(const SpmmHostDesc& d, const SpmmWsLayout& L, char* ws, const float* B,
                 int64_t ldb, int32_t col0, int32_t fw, uint32_t kmax, float* C, int64_t ldc,
                 int32_t accumulate, int32_t f_total, hipStream_t s, const SweepFusedArgs* fused, int32_t fuse) {
  if (d.n_waves <= 0) return SAGNN_OK;
  const SweepFusedArgs fa = fused ? *fused : SweepFusedArgs{};
  if (!fused) fuse = 0;
  SweepDims sd{};
  sd.n_waves = d.n_waves; sd.ldb = ldb; sd.ldc = ldc; sd.f_total = f_total;
  sd.generation = d.generation; sd.col0 = col0; sd.accumulate = accumulate;
  // bytes of B reachable from B + col0: rows 0..kmax, fw columns each (columns were clamped to
  // kmax when the stream was built)
  sd.b_bytes = 0;
  const bool buf = buffer_addressable(kmax, ldb, fw, &sd.b_bytes);
  sd.row_bytes = (uint32_t)(ldb * 4);
  const unsigned blocks = (unsigned)ceil_div(d.n_waves, 4);
  sd.slots = d.slots > 0 && d.slots <= kSweepSlots ? d.slots : kSweepSlots;
  const size_t lds = (size_t)4 * sd.slots * fw * sizeof(float);
  auto go = [&](auto kern) -> int {
    if (lds > 48 * 1024)
      SAGNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), lds, s,
                       reinterpret_cast<const uint32_t*>(ws + L.code),
                       reinterpret_cast<const float*>(ws + L.vals),
                       reinterpret_cast<const int32_t*>(ws + L.wave_base),
                       reinterpret_cast<const int32_t*>(ws + L.piece_target),
                       reinterpret_cast<const SpmmWsHeader*>(ws + L.header), B + col0, C + col0,
                       reinterpret_cast<float*>(ws + L.partial), sd);
    SAGNN_LAUNCH_CHECK();
    return SAGNN_OK;
  };
  // lane-group kernels: walk the stream interval by interval, with a barrier of the XCD's
  // resident workgroups in between when the schedule was laid out for it
  auto go_group = [&](auto kern) -> int {
    if (lds > 48 * 1024)
      SAGNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    uint32_t* barrier = reinterpret_cast<uint32_t*>(ws + L.barrier);
    sd.n_intervals = d.n_intervals > 0 ? d.n_intervals : 1;
    sd.sync_timeout_ticks = d.sync_timeout_ticks;
    sd.sync_test_extra = d.sync_test_extra;
    sd.wg_per_cohort = 0;
    sd.pace_ticks = d.barriers ? 0.f : (float)d.pace_ps_per_step * 1e-4f;    // ps -> 10 ns ticks
    if (d.barriers && d.sync_slabs > 0 && sd.n_intervals > 1 && (d.n_waves & 3) == 0) {
      const int wpc = resident_workgroups(reinterpret_cast<const void*>(kern), lds);
      const int64_t cohorts = wpc > 0 ? ceil_div((int64_t)blocks, wpc) : 0;
      if (wpc >= 8 && cohorts * 8 * sd.n_intervals <= kSweepBarrierSlots) {
        sd.wg_per_cohort = wpc;
        const int n_ctr = (int)(cohorts * 8 * sd.n_intervals);
        hipLaunchKernelGGL(sweep_barrier_clear_kernel, dim3((unsigned)ceil_div(n_ctr, 256)), dim3(256), 0, s,
                           barrier, n_ctr);
        SAGNN_LAUNCH_CHECK();
      }
    }
    if (sd.wg_per_cohort == 0) sd.n_intervals = sd.n_intervals > 1 ? -sd.n_intervals : sd.n_intervals;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), lds, s,
                       reinterpret_cast<const uint32_t*>(ws + L.code),
                       reinterpret_cast<const float*>(ws + L.vals),
                       reinterpret_cast<const int32_t*>(ws + L.wave_base),
                       reinterpret_cast<const int32_t*>(ws + L.piece_target),
                       reinterpret_cast<const SpmmWsHeader*>(ws + L.header), B + col0, C + col0,
                       reinterpret_cast<float*>(ws + L.partial),
                       reinterpret_cast<const int32_t*>(ws + L.sync_off), barrier,
                       reinterpret_cast<const float*>(ws + L.sched), sd, fa);
    SAGNN_LAUNCH_CHECK();
    return SAGNN_OK;
  };
  if (fuse != 0 && d.groups != 2 && d.groups != 4) return SAGNN_EINVAL;   // (groups == 1: sweep_launch_fused)
  if (d.groups == 16)    // prepared for f = 16: four lanes per row
    return fw == 16 ? (buf ? go(spmm_sweep_perm_kernel<16, true>) : go(spmm_sweep_perm_kernel<16, false>))
                    : SAGNN_EINVAL;
  if (d.groups == 8)     // prepared for f = 32: eight lanes per row
    return fw == 32 ? (buf ? go(spmm_sweep_perm_kernel<8, true>) : go(spmm_sweep_perm_kernel<8, false>))
                    : SAGNN_EINVAL;
  if (d.groups == 2) {   // prepared for f = 128: half a wavefront per row (or per half row at 64)
    if (fw == 128) return buf ? go_group(group_kernel_of<4, 2, true>(fuse)) : go_group(group_kernel_of<4, 2, false>(fuse));
    if (fw == 64) return buf ? go_group(group_kernel_of<2, 2, true>(fuse)) : go_group(group_kernel_of<2, 2, false>(fuse));
    return SAGNN_EINVAL;
  }
  if (d.groups == 4) {   // prepared for f = 64: a quarter wavefront per row
    if (fw == 64) return buf ? go_group(group_kernel_of<4, 4, true>(fuse)) : go_group(group_kernel_of<4, 4, false>(fuse));
    return SAGNN_EINVAL;
  }
  if (fw == 256) return buf ? go(spmm_sweep_kernel<4, 8, true>) : go(spmm_sweep_kernel<4, 8, false>);
  if (fw == 128) return buf ? go(spmm_sweep_kernel<2, 8, true>) : go(spmm_sweep_kernel<2, 8, false>);
  if (fw == 64) return buf ? go(spmm_sweep_kernel<1, 8, true>) : go(spmm_sweep_kernel<1, 8, false>);
  return SAGNN_EINVAL;
}

int sweep_launch_fused(const SpmmHostDesc& d, const SpmmWsLayout& L, char* ws, const float* B, int64_t ldb,
                       int32_t f_in, uint32_t kmax, const SweepFusedArgs& fa, int32_t mode, hipStream_t s) {
  if (d.n_waves <= 0 || (d.n_waves & 3) || d.slots != kSweepSlots) return SAGNN_EINVAL;
  if (mode < 0 || mode > 2) return SAGNN_EINVAL;
  if (!(f_in == 64 || f_in == 128 || f_in == 256) || fa.f_out <= 0 || fa.f_out > 256 || !fa.W) return SAGNN_EINVAL;
  if (d.groups == 2 || d.groups == 4) {
    // lane-group schedules: the same kernels as the product, with the dense transform compiled in
    SweepFusedArgs fg = fa;
    fg.Wp = nullptr;
    if (mode != 0) {
      const int32_t NB = (fa.f_out + 31) / 32 * 32;
      __bf16* wp = reinterpret_cast<__bf16*>(ws + L.wpack);
      hipLaunchKernelGGL(sweep_pack_w_kernel, dim3((unsigned)ceil_div((int64_t)(f_in / 8) * NB, 256)), dim3(256), 0, s,
                         fa.W, f_in, fa.f_out, NB, wp, mode == 2 ? 3 : 1);
      SAGNN_LAUNCH_CHECK();
      fg.Wp = wp;
    }
    return sweep_launch(d, L, ws, B, ldb, 0, f_in, kmax, nullptr, f_in, 0, f_in, s, &fg, mode + 1);
  }
  if (d.groups != 1) return SAGNN_EINVAL;
  SweepDims sd{};
  sd.n_waves = d.n_waves; sd.ldb = ldb; sd.ldc = f_in; sd.f_total = f_in;
  sd.generation = d.generation; sd.col0 = 0; sd.accumulate = 0; sd.slots = kSweepSlots;
  sd.b_bytes = 0;
  const bool buf = buffer_addressable(kmax, ldb, f_in, &sd.b_bytes);
  sd.row_bytes = (uint32_t)(ldb * 4);
  const unsigned blocks = (unsigned)(d.n_waves / 4);
  const size_t lds = (size_t)4 * kSweepSlots * f_in * sizeof(float);
  SweepFusedArgs fb = fa;
  fb.Wp = nullptr;
  if (mode != 0) {
    const int32_t NB = (fa.f_out + 31) / 32 * 32;
    __bf16* wp = reinterpret_cast<__bf16*>(ws + L.wpack);
    hipLaunchKernelGGL(sweep_pack_w_kernel, dim3((unsigned)ceil_div((int64_t)(f_in / 8) * NB, 256)), dim3(256), 0, s,
                       fa.W, f_in, fa.f_out, NB, wp, mode == 2 ? 3 : 1);
    SAGNN_LAUNCH_CHECK();
    fb.Wp = wp;
  }
  auto go = [&](auto kern) -> int {
    if (lds > 48 * 1024)
      SAGNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), lds, s,
                       reinterpret_cast<const uint32_t*>(ws + L.code),
                       reinterpret_cast<const float*>(ws + L.vals),
                       reinterpret_cast<const int32_t*>(ws + L.wave_base),
                       reinterpret_cast<const int32_t*>(ws + L.piece_target),
                       reinterpret_cast<const SpmmWsHeader*>(ws + L.header), B,
                       reinterpret_cast<float*>(ws + L.partial), sd, fb);
    SAGNN_LAUNCH_CHECK();
    return SAGNN_OK;
  };
#define SAGNN_SWF(FPL_)                                                                                      \
  (mode == 2 ? (buf ? go(spmm_sweep_fused_kernel<FPL_, 8, true, 2>) : go(spmm_sweep_fused_kernel<FPL_, 8, false, 2>))   \
   : mode == 1 ? (buf ? go(spmm_sweep_fused_kernel<FPL_, 8, true, 1>) : go(spmm_sweep_fused_kernel<FPL_, 8, false, 1>)) \
               : (buf ? go(spmm_sweep_fused_kernel<FPL_, 8, true, 0>) : go(spmm_sweep_fused_kernel<FPL_, 8, false, 0>)))
  if (f_in == 256) return SAGNN_SWF(4);
  if (f_in == 128) return SAGNN_SWF(2);
  return SAGNN_SWF(1);
#undef SAGNN_SWF
}

int sweep_combine(const SpmmHostDesc& d, const SpmmWsLayout& L, char* ws, float* C, int64_t ldc,
                  int32_t f_total, int32_t accumulate, hipStream_t s) {
  if (d.n_multi_rows <= 0) return SAGNN_OK;
  hipLaunchKernelGGL(sweep_combine_kernel, dim3((unsigned)ceil_div(d.n_multi_rows, 4)), dim3(256), 0, s,
                     reinterpret_cast<const int32_t*>(ws + L.multi_row),
                     reinterpret_cast<const int32_t*>(ws + L.multi_first),
                     reinterpret_cast<const float*>(ws + L.partial),
                     reinterpret_cast<const SpmmWsHeader*>(ws + L.header), d.generation, d.n_multi_rows,
                     C, ldc, f_total, accumulate);
  SAGNN_LAUNCH_CHECK();
  return SAGNN_OK;
}

}  // namespace sagnn
