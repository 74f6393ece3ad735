// Needed-row planning: NnzCols of every column block of a CSR row block (Sec. 4.1, the
// paragraph that defines NnzCols(i,j) as the nonzero column indices of block A_ij, i.e. the
// rows of H_j that P(i) has to receive).
//
// Integer only, result unique.  Pipeline (all kernels on the caller's stream):
//   clear    one flag byte per column
//   mark     one pass over colidx: flag[c] = 1.  Plain byte stores: every writer stores the
//            same value, so no atomics are needed, and a test before the store keeps hub
//            columns from producing write traffic at all
//   words    a lane squeezes 16 flag bytes (one 16-byte load) into 16 bits, four lanes make the
//            64-bit membership word of 64 columns; its popcount feeds the scan
//   scan     exclusive scan of the per-block popcounts (one workgroup)       \  three-kernel
//   prefix   per-word exclusive prefix = rank of the word's first column       /  scan
//   blkoff   rank of every column-block boundary -> blk_off, N   (then one D2H copy + sync)
//   emit     one wavefront per word: lane l owns column 64w+l, the ballot mask and mbcnt give
//            each set lane its slot (ballot / prefix-count stream compaction); needed[] comes
//            out ascending
//   remap    compact[e] = prefix[c>>6] + popcount(word & bits below c): position of column
//            c in needed[]; monotone in c, so sorted rows stay sorted
// Traffic: nnz*4 (mark) + nnz*8 (remap read+write) + N*4 + a few passes over n bytes.
#include <mutex>

#include "common.h"

namespace sagnn {
namespace {

constexpr int kThreads = 256;
constexpr int kWordsPerBlock = 2048;  // scan tile: 256 threads x 8 words

// LDS marking (column ranges small enough to be covered by a few LDS-resident bitmaps):
// a workgroup owns a private bitmap of kLdsCols columns in LDS and a share of the entries.
constexpr int kLdsThreads = 1024;
constexpr int kLdsWords = 38912;                    // 32-bit words: 152 KB of the CU's 160 KB
constexpr int64_t kLdsCols = (int64_t)kLdsWords * 32;
constexpr int kLdsMaxPasses = 4;
constexpr int kLdsGroups = 256;                     // workgroups in total (one per CU)
constexpr int64_t kLdsMinNnz = 1ll << 22;

inline bool lds_mark_eligible(int64_t n, int64_t nnz) {
  return nnz >= kLdsMinNnz && n > 0 && n <= kLdsMaxPasses * kLdsCols;
}

// Wider column ranges: the entries are first partitioned by column range (count, offsets, scatter:
// streaming passes over colidx with LDS counters), then every range is marked from its own bucket
// by one workgroup whose LDS holds one flag BYTE per column (plain stores: LDS atomics run at about
// one lane per five clocks, a bit per column would cost more than the byte flags in memory do) and
// which turns the bytes into the range's membership words itself.  Byte flags in memory cost one
// cache-line fill per entry; this costs three streaming passes.
constexpr int64_t kBktCols = 155648;                // columns per range: 152 KB of flag bytes, a multiple of 64
constexpr int kBktMaxRanges = 2048;
constexpr int kBktGroups = 256;                     // workgroups of the partition passes
constexpr int kBktThreads = 1024;                   // their size: 16 wavefronts keep enough loads in flight
inline int64_t bucket_ranges(int64_t n) { return ceil_div(n > 0 ? n : 1, kBktCols); }
inline bool bucket_mark_eligible(int64_t n, int64_t nnz) {
  return nnz >= kLdsMinNnz && n > kLdsMaxPasses * kLdsCols && bucket_ranges(n) <= kBktMaxRanges;
}

struct PlanWs {
  uint8_t* flag;      // n bytes (rounded up to 64W)
  uint64_t* bitmap;   // W words
  int32_t* prefix;    // W + 1
  uint4* rank16;      // W: {word lo, word hi, prefix, 0}: one 16-byte lookup per remapped entry
  int32_t* blocksum;  // nblk + 1
  int64_t* colblk;    // nb + 1 (device copy of the block boundaries)
  int64_t* blkoff;    // nb + 1
  int32_t* err;       // 4 counters
  uint32_t* part;     // LDS marking only: kLdsGroups private bitmaps of kLdsWords words
  int32_t* bkt_cols;  // bucketed marking only: the column ids partitioned by range (nnz)
  int32_t* bkt_place; // bucketed marking only: where in bkt_cols every entry went (nnz; -1: column out of range)
  int32_t* bkt_cnt;   // bucketed marking only: [ranges][kBktGroups] counts, then offsets inside the range
  int32_t* bkt_start; // bucketed marking only: first entry of every range (+ total)
  int64_t W, nblk;
  size_t bytes;
};

PlanWs carve(void* base, int64_t n, int32_t nb, int64_t nnz) {
  PlanWs w;
  w.W = ceil_div(n > 0 ? n : 1, 64);
  w.nblk = ceil_div(w.W, kWordsPerBlock);
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off += round_up(bytes, 256);
    return reinterpret_cast<char*>(base) + o;
  };
  w.flag = reinterpret_cast<uint8_t*>(take((size_t)w.W * 64));
  w.bitmap = reinterpret_cast<uint64_t*>(take(sizeof(uint64_t) * (size_t)w.W));
  w.prefix = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * (size_t)(w.W + 1)));
  w.rank16 = reinterpret_cast<uint4*>(take(sizeof(uint4) * (size_t)w.W));
  w.blocksum = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * (size_t)(w.nblk + 1)));
  w.colblk = reinterpret_cast<int64_t*>(take(sizeof(int64_t) * (size_t)(nb + 1)));
  w.blkoff = reinterpret_cast<int64_t*>(take(sizeof(int64_t) * (size_t)(nb + 1)));
  w.err = reinterpret_cast<int32_t*>(take(256));   // 4 counters; the small-block path keeps its result record here
  const bool bucketed = bucket_mark_eligible(n, nnz);
  w.part = lds_mark_eligible(n, nnz)
               ? reinterpret_cast<uint32_t*>(take(sizeof(uint32_t) * (size_t)kLdsGroups * kLdsWords))
               : nullptr;
  w.bkt_cols = bucketed ? reinterpret_cast<int32_t*>(take(sizeof(int32_t) * (size_t)nnz)) : nullptr;
  w.bkt_place = bucketed ? reinterpret_cast<int32_t*>(take(sizeof(int32_t) * (size_t)nnz)) : nullptr;
  w.bkt_cnt = bucketed ? reinterpret_cast<int32_t*>(take(sizeof(int32_t) * (size_t)(bucket_ranges(n) * kBktGroups)))
                       : nullptr;
  w.bkt_start = bucketed ? reinterpret_cast<int32_t*>(take(sizeof(int32_t) * (size_t)(bucket_ranges(n) + 1))) : nullptr;
  w.bytes = off;
  return w;
}

__device__ __forceinline__ int64_t ceil_div_dev(int64_t a, int64_t b) { return (a + b - 1) / b; }

__global__ __launch_bounds__(kThreads) void clear_kernel(uint4* __restrict__ flag16, int64_t n16,
                                                         int32_t* __restrict__ err) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n16; i += stride)
    flag16[i] = make_uint4(0u, 0u, 0u, 0u);
  if (blockIdx.x == 0 && threadIdx.x < 4) err[threadIdx.x] = 0;
}

// Sparsity-oblivious plan: every column of [0, n) counts as needed (the whole block row of H
// is transferred, Sec. 4.1 "sparsity-oblivious algorithm"); bytes past n stay clear.
__global__ __launch_bounds__(kThreads) void fill_all_kernel(uint8_t* __restrict__ flag, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t c = (int64_t)blockIdx.x * kThreads + threadIdx.x; c < n; c += stride) flag[c] = 1;
}

// err[0]: rowptr malformed, err[1]: column out of range
__global__ __launch_bounds__(kThreads) void validate_rowptr_kernel(
    const int32_t* __restrict__ rowptr, int64_t m, int64_t nnz, int32_t* __restrict__ err) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t r = (int64_t)blockIdx.x * kThreads + threadIdx.x; r < m; r += stride)
    if (rowptr[r] > rowptr[r + 1]) err[0] = 1;
  if (blockIdx.x == 0 && threadIdx.x == 0)
    if (rowptr[0] != 0 || (int64_t)rowptr[m] != nnz) err[0] = 1;
}

__device__ __forceinline__ void mark_one(int32_t c, int64_t n, uint8_t* __restrict__ flag,
                                         int32_t* __restrict__ err) {
  if (c < 0 || c >= n) {
    err[1] = 1;
    return;
  }
  // benign race: all writers store 1.  Testing first is measurably faster than storing
  // unconditionally on power-law graphs (hub columns are hit thousands of times).
  if (flag[c] == 0) flag[c] = 1;
}

// 4 entries per thread per iteration (16-byte loads when the index array is aligned).  (Issuing
// the probes of eight entries before the first store was measured slower: 546 against 517 us on
// 27 M entries over 111 M columns -- the kernel is bound by the line fills, not by their latency.)
__global__ __launch_bounds__(kThreads) void mark_kernel(const int32_t* __restrict__ colidx,
                                                        int64_t nnz, int64_t n,
                                                        uint8_t* __restrict__ flag,
                                                        int32_t* __restrict__ err, int aligned) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  const int64_t quads = nnz >> 2;
  if (aligned) {
    const int4* __restrict__ c4 = reinterpret_cast<const int4*>(colidx);
    for (int64_t q = (int64_t)blockIdx.x * kThreads + threadIdx.x; q < quads; q += stride) {
      const int4 c = c4[q];
      mark_one(c.x, n, flag, err);
      mark_one(c.y, n, flag, err);
      mark_one(c.z, n, flag, err);
      mark_one(c.w, n, flag, err);
    }
    for (int64_t e = (quads << 2) + (int64_t)blockIdx.x * kThreads + threadIdx.x; e < nnz; e += stride)
      mark_one(colidx[e], n, flag, err);
  } else {
    for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < nnz; e += stride)
      mark_one(colidx[e], n, flag, err);
  }
}

// --- LDS marking ---------------------------------------------------------------------------
// Byte probes into a flag array cost one cache-line fill each (the array is far larger than
// a CU's L1), which is what bounds mark_kernel.  When a few LDS-sized bitmaps cover all
// columns, a workgroup instead ORs the bits of its share of the entries into a private LDS
// bitmap of one column range (pass), reading colidx once per pass as a stream, and writes
// the bitmap out; merge_kernel ORs the private bitmaps into the membership words.
__device__ __forceinline__ void lds_mark_one(int32_t c, int64_t n, int64_t c0, uint32_t* bits,
                                             int32_t* __restrict__ err) {
  if (c < 0 || c >= n) {
    err[1] = 1;
    return;
  }
  const int64_t rel = (int64_t)c - c0;
  if (rel >= 0 && rel < kLdsCols) {
    // test first: lanes that read one address are served by a broadcast, lanes that update one
    // address are serialised, and hub columns come up thousands of times
    const uint32_t bit = 1u << (rel & 31);
    if ((__hip_atomic_load(&bits[rel >> 5], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) & bit) == 0)
      __hip_atomic_fetch_or(&bits[rel >> 5], bit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  }
}

// `spec` (may be NULL): the workgroups of the first column range also write the range-checked
// copy of colidx that the remap is if every column turns out to be needed (a whole graph planned
// as one block): the entries are in registers anyway, and the separate copy pass is then skipped.
__device__ __forceinline__ int32_t identity_or_bad(int32_t c, int64_t n) { return (c < 0 || c >= n) ? -1 : c; }

__global__ __launch_bounds__(kLdsThreads) void mark_lds_kernel(const int32_t* __restrict__ colidx,
                                                               int64_t nnz, int64_t n,
                                                               int32_t groups_per_pass,
                                                               uint32_t* __restrict__ part,
                                                               int32_t* __restrict__ err, int aligned,
                                                               int32_t* __restrict__ spec) {
  extern __shared__ __attribute__((aligned(16))) uint32_t bits[];
  const int pass = blockIdx.x / groups_per_pass, share = blockIdx.x % groups_per_pass;
  if (pass != 0) spec = nullptr;
  const int64_t c0 = (int64_t)pass * kLdsCols;
  uint4* b4 = reinterpret_cast<uint4*>(bits);
  for (int i = threadIdx.x; i < kLdsWords / 4; i += kLdsThreads) b4[i] = make_uint4(0u, 0u, 0u, 0u);
  __syncthreads();
  if (aligned) {
    const int64_t quads = nnz >> 2;
    const int64_t per = ceil_div_dev(quads, groups_per_pass);
    const int64_t q0 = (int64_t)share * per;
    const int64_t q1 = q0 + per < quads ? q0 + per : quads;
    const int4* __restrict__ c4 = reinterpret_cast<const int4*>(colidx);
    // four independent 16-byte loads per thread in flight (the scan is a pure stream)
    int64_t q = q0 + threadIdx.x;
    for (; q + 3 * kLdsThreads < q1; q += 4 * kLdsThreads) {
      int4 c[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) c[j] = c4[q + j * kLdsThreads];
      if (spec) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          reinterpret_cast<int4*>(spec)[q + j * kLdsThreads] =
              make_int4(identity_or_bad(c[j].x, n), identity_or_bad(c[j].y, n), identity_or_bad(c[j].z, n),
                        identity_or_bad(c[j].w, n));
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        lds_mark_one(c[j].x, n, c0, bits, err);
        lds_mark_one(c[j].y, n, c0, bits, err);
        lds_mark_one(c[j].z, n, c0, bits, err);
        lds_mark_one(c[j].w, n, c0, bits, err);
      }
    }
    for (; q < q1; q += kLdsThreads) {
      const int4 c = c4[q];
      if (spec)
        reinterpret_cast<int4*>(spec)[q] = make_int4(identity_or_bad(c.x, n), identity_or_bad(c.y, n),
                                                     identity_or_bad(c.z, n), identity_or_bad(c.w, n));
      lds_mark_one(c.x, n, c0, bits, err);
      lds_mark_one(c.y, n, c0, bits, err);
      lds_mark_one(c.z, n, c0, bits, err);
      lds_mark_one(c.w, n, c0, bits, err);
    }
    if (share == 0)
      for (int64_t e = (quads << 2) + threadIdx.x; e < nnz; e += kLdsThreads) {
        const int32_t c = colidx[e];
        if (spec) spec[e] = identity_or_bad(c, n);
        lds_mark_one(c, n, c0, bits, err);
      }
  } else {
    const int64_t per = ceil_div_dev(nnz, groups_per_pass);
    const int64_t e0 = (int64_t)share * per;
    const int64_t e1 = e0 + per < nnz ? e0 + per : nnz;
    for (int64_t e = e0 + threadIdx.x; e < e1; e += kLdsThreads) {
      const int32_t c = colidx[e];
      if (spec) spec[e] = identity_or_bad(c, n);
      lds_mark_one(c, n, c0, bits, err);
    }
  }
  __syncthreads();
  // only the words that cover columns below n are ever read back
  const int64_t cols_here = n - c0 < kLdsCols ? n - c0 : kLdsCols;
  const int used4 = cols_here > 0 ? (int)((cols_here + 127) >> 7) : 0;
  uint4* __restrict__ out = reinterpret_cast<uint4*>(part + (size_t)blockIdx.x * kLdsWords);
  for (int i = threadIdx.x; i < used4; i += kLdsThreads) out[i] = b4[i];
}

// --- bucketed marking ------------------------------------------------------------------------
// entries of workgroup g: [g * per, (g + 1) * per); cnt[b * kBktGroups + g] = its entries in range b
//
// Columns are ascending inside a row, so neighbouring lanes often fall into the same range (about
// 13 of 64 lanes share one on an R-MAT block) and their LDS atomics on one counter would run one
// after the other.  A run of equal ranges in adjacent lanes is therefore counted by its first lane
// alone: heads = lanes whose lower neighbour differs, the run's length comes from the ballot of heads.
struct LaneRun {
  int head;    // first lane of this lane's run
  int len;     // length of the run (meaningful in its first lane)
  bool first;
};
__device__ __forceinline__ LaneRun lane_run(int32_t b, int lane) {
  const int32_t prev = __shfl_up(b, 1, 64);
  LaneRun r;
  r.first = lane == 0 || prev != b;
  const uint64_t heads = __ballot(r.first);
  r.head = 63 - __clzll((long long)(heads & (~0ull >> (63 - lane))));
  const uint64_t above = lane == 63 ? 0ull : heads >> (lane + 1);
  r.len = above ? __ffsll((long long)above) : 64 - lane;
  return r;
}

// per workgroup: how many of its entries fall into every range (out-of-range columns are flagged and left out)
__global__ __launch_bounds__(kBktThreads) void bucket_count_kernel(const int32_t* __restrict__ colidx, int64_t nnz,
                                                                int64_t n, int32_t nbk, int32_t* __restrict__ cnt,
                                                                int32_t* __restrict__ err) {
  __shared__ int32_t h[kBktMaxRanges];
  for (int b = threadIdx.x; b < nbk; b += kBktThreads) h[b] = 0;
  __syncthreads();
  const int lane = threadIdx.x & 63;
  const int64_t per = ceil_div_dev(nnz, kBktGroups);
  const int64_t e0 = (int64_t)blockIdx.x * per, e1 = e0 + per < nnz ? e0 + per : nnz;
  // eight independent loads per thread in flight; the trip count is the same for every lane (ballots inside)
  for (int64_t base = e0; base < e1; base += 8 * kBktThreads) {
    const int64_t e = base + threadIdx.x;
    int32_t c[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) c[j] = e + j * kBktThreads < e1 ? colidx[e + j * kBktThreads] : 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      int32_t b = -1;                                    // past the end or out of range: no bucket
      if (e + j * kBktThreads < e1) {
        if (c[j] < 0 || c[j] >= n) err[1] = 1;
        else b = (int32_t)((uint32_t)c[j] / (uint32_t)kBktCols);
      }
      const LaneRun r = lane_run(b, lane);
      if (r.first && b >= 0) atomicAdd(&h[b], r.len);
    }
  }
  __syncthreads();
  for (int b = threadIdx.x; b < nbk; b += kBktThreads) cnt[(int64_t)b * kBktGroups + blockIdx.x] = h[b];
}

// one workgroup per range: the counts of the kBktGroups workgroups become offsets inside the
// range, the range's total goes to tot[range]
__global__ __launch_bounds__(kBktGroups) void bucket_within_kernel(int32_t* __restrict__ cnt, int32_t* __restrict__ tot) {
  __shared__ int32_t wsum[kBktGroups / 64];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int32_t* __restrict__ c = cnt + (int64_t)blockIdx.x * kBktGroups;
  const int32_t v = c[threadIdx.x];
  int32_t inc = v;
  for (int o = 1; o < 64; o <<= 1) {
    const int32_t t = __shfl_up(inc, o, 64);
    if (lane >= o) inc += t;
  }
  if (lane == 63) wsum[w] = inc;
  __syncthreads();
  int32_t before = 0;
  for (int j = 0; j < w; ++j) before += wsum[j];
  c[threadIdx.x] = before + inc - v;
  if (threadIdx.x == kBktGroups - 1) tot[blockIdx.x] = before + inc;
}

// exclusive scan in place of the range totals (nbk <= kBktMaxRanges), grand total to a[nbk]; one workgroup
__global__ __launch_bounds__(1024) void bucket_starts_kernel(int32_t* __restrict__ a, int32_t nbk) {
  __shared__ int32_t wsum[16];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int i0 = threadIdx.x * 2;
  const int32_t v0 = i0 < nbk ? a[i0] : 0, v1 = i0 + 1 < nbk ? a[i0 + 1] : 0;
  int32_t inc = v0 + v1;
  for (int o = 1; o < 64; o <<= 1) {
    const int32_t t = __shfl_up(inc, o, 64);
    if (lane >= o) inc += t;
  }
  if (lane == 63) wsum[w] = inc;
  __syncthreads();
  int32_t before = 0;
  for (int j = 0; j < w; ++j) before += wsum[j];
  const int32_t excl = before + inc - v0 - v1;
  __syncthreads();
  if (i0 < nbk) a[i0] = excl;
  if (i0 + 1 < nbk) a[i0 + 1] = excl + v0;
  if (threadIdx.x == 1023) a[nbk] = before + inc;
}

// Every workgroup places its entries behind its own offset of every range.  A batch of 8192 entries
// is first sorted by range inside LDS (count per range, scan, place; runs of adjacent lanes with one
// range share one atomic) and then written out in that order, so that neighbouring lanes store to
// neighbouring places of one range (about a dozen entries per range and batch on a wide block)
// instead of to as many ranges as there are lanes.
constexpr int kBktBatch = 8 * kBktThreads;
__global__ __launch_bounds__(kBktThreads) void bucket_scatter_kernel(const int32_t* __restrict__ colidx, int64_t nnz,
                                                                  int64_t n, int32_t nbk,
                                                                  const int32_t* __restrict__ within,
                                                                  const int32_t* __restrict__ start,
                                                                  int32_t* __restrict__ cols,
                                                                  int32_t* __restrict__ place_e) {
  __shared__ int32_t off[kBktMaxRanges];   // this workgroup's next free place in every range
  __shared__ int32_t cur[kBktMaxRanges];   // batch: entries per range
  __shared__ int32_t cs[kBktMaxRanges];    // batch: first staged position of every range
  __shared__ int32_t stage[kBktBatch];
  __shared__ int32_t wsum[kBktThreads / 64];
  static_assert(kBktMaxRanges == 2 * kBktThreads, "a thread scans two ranges");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b0 = 2 * tid, b1 = 2 * tid + 1;                      // the two ranges this thread keeps
  off[b0] = b0 < nbk ? start[b0] + within[(int64_t)b0 * kBktGroups + blockIdx.x] : 0;
  off[b1] = b1 < nbk ? start[b1] + within[(int64_t)b1 * kBktGroups + blockIdx.x] : 0;
  cur[b0] = 0;
  cur[b1] = 0;
  __syncthreads();
  const int64_t per = ceil_div_dev(nnz, kBktGroups);
  const int64_t e0 = (int64_t)blockIdx.x * per, e1 = e0 + per < nnz ? e0 + per : nnz;
  for (int64_t base = e0; base < e1; base += kBktBatch) {
    const int64_t e = base + tid;
    int32_t c[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) c[j] = e + j * kBktThreads < e1 ? colidx[e + j * kBktThreads] : -1;
    // count per range; the value an atomic returns is the entry's place among its range's entries of
    // this batch, so one pass of LDS atomics (about one lane per clock) serves both the counts and the order
    int32_t b[8], rank[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      b[j] = (c[j] < 0 || c[j] >= n) ? -1 : (int32_t)((uint32_t)c[j] / (uint32_t)kBktCols);
      const LaneRun r = lane_run(b[j], lane);
      int32_t first_rank = 0;
      if (r.first && b[j] >= 0) first_rank = atomicAdd(&cur[b[j]], r.len);
      rank[j] = __shfl(first_rank, r.head, 64) + (lane - r.head);
    }
    __syncthreads();
    // exclusive scan of the counts: cs = first staged position of a range
    const int v0 = cur[b0], v1 = cur[b1];
    int inc = v0 + v1;
    for (int o = 1; o < 64; o <<= 1) {
      const int t = __shfl_up(inc, o, 64);
      if (lane >= o) inc += t;
    }
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kBktThreads / 64; ++w) {
      if (w < wave) before += wsum[w];
      total += wsum[w];
    }
    const int ex = before + inc - (v0 + v1);
    cs[b0] = ex;
    cs[b1] = ex + v0;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      // (the order inside a range does not matter: the marks are a set)
      if (b[j] >= 0) {
        const int32_t pos = cs[b[j]] + rank[j];
        if (pos >= 0 && pos < kBktBatch) stage[pos] = c[j];
      }
      // where the entry ends up in the partitioned array (the remap finds its rank there)
      if (place_e && e + j * kBktThreads < e1) place_e[e + j * kBktThreads] = b[j] >= 0 ? off[b[j]] + rank[j] : -1;
    }
    __syncthreads();
    for (int i = tid; i < total; i += kBktThreads) {
      const int32_t col = stage[i];
      const int32_t rb = (int32_t)((uint32_t)col / (uint32_t)kBktCols);
      const int64_t place = (int64_t)off[rb] + (i - cs[rb]);
      if (place >= 0 && place < nnz) cols[place] = col;
    }
    __syncthreads();
    off[b0] += cur[b0];
    off[b1] += cur[b1];
    cur[b0] = 0;
    cur[b1] = 0;
    __syncthreads();
  }
}

// The remap of a wide block from the partitioned entries.  Looked up in entry order, every rank
// costs a line of a table that no L2 holds (27.7 MB of rank records for 111 M columns).  In range
// order the records of one range (39 KB) sit in LDS: a workgroup per range replaces every
// column id of its bucket by the column's rank, in place; the entries then fetch their rank from
// the place the scatter noted for them.  That gather is local: a workgroup's share of the entries
// went to its own segment of every range, a few lines per range that stay in L2 while the share
// is walked.
__global__ __launch_bounds__(kLdsThreads) void remap_bucket_kernel(int32_t* __restrict__ cols,
                                                                   const int32_t* __restrict__ start, int64_t nnz,
                                                                   int64_t n, int64_t W,
                                                                   const uint4* __restrict__ rank16) {
  // per 32 columns: {membership bits, needed columns before them}: a lookup is one 8-byte LDS read
  __shared__ uint2 rec[kBktCols / 32];
  const int range = blockIdx.x;
  const int64_t w0 = (int64_t)range * (kBktCols / 64);
  for (int i = threadIdx.x; i < (int)(kBktCols / 64); i += kLdsThreads) {
    const uint4 t = w0 + i < W ? rank16[w0 + i] : make_uint4(0u, 0u, 0u, 0u);
    rec[2 * i] = make_uint2(t.x, t.z);
    rec[2 * i + 1] = make_uint2(t.y, t.z + (uint32_t)__popc(t.x));
  }
  __syncthreads();
  const int64_t c0 = (int64_t)range * kBktCols;
  int64_t e0 = start[range], e1 = start[range + 1];
  e0 = e0 < 0 ? 0 : e0;
  e1 = e1 > nnz ? nnz : e1;
  for (int64_t e = e0 + threadIdx.x; e < e1; e += 8 * kLdsThreads) {
    int32_t c[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) c[j] = e + j * kLdsThreads < e1 ? cols[e + j * kLdsThreads] : -1;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (e + j * kLdsThreads >= e1) continue;
      const int64_t rel = (int64_t)c[j] - c0;
      int32_t rk = -1;
      if (rel >= 0 && rel < kBktCols && c[j] < n) {
        const uint2 t = rec[rel >> 5];
        rk = (int32_t)t.y + __popc(t.x & ((1u << (rel & 31)) - 1u));
      }
      cols[e + j * kLdsThreads] = rk;
    }
  }
}

// compact[e] = rank found at the entry's place (same shares of the entries as the scatter)
__global__ __launch_bounds__(kBktThreads) void remap_gather_kernel(const int32_t* __restrict__ place_e,
                                                                  const int32_t* __restrict__ ranks, int64_t nnz,
                                                                  int32_t* __restrict__ compact) {
  const int64_t per = ceil_div_dev(nnz, kBktGroups);
  const int64_t e0 = (int64_t)blockIdx.x * per, e1 = e0 + per < nnz ? e0 + per : nnz;
  for (int64_t e = e0 + threadIdx.x; e < e1; e += 8 * kBktThreads) {
    int32_t p[8], r[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) p[j] = e + j * kBktThreads < e1 ? __builtin_nontemporal_load(&place_e[e + j * kBktThreads]) : -1;
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = (p[j] >= 0 && p[j] < nnz) ? ranks[p[j]] : -1;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (e + j * kBktThreads < e1) __builtin_nontemporal_store(r[j], &compact[e + j * kBktThreads]);
  }
}

// one workgroup per range: flag bytes in LDS from the range's bucket, then the range's membership
// words (kBktCols / 64 of them, the last range fewer) straight into the bitmap
__global__ __launch_bounds__(kLdsThreads) void mark_bucket_kernel(const int32_t* __restrict__ cols,
                                                                  const int32_t* __restrict__ start, int64_t nnz,
                                                                  int64_t n, int64_t W, uint64_t* __restrict__ bm) {
  extern __shared__ __attribute__((aligned(16))) uint32_t bits[];
  uint8_t* flag = reinterpret_cast<uint8_t*>(bits);
  const int range = blockIdx.x;
  const int64_t c0 = (int64_t)range * kBktCols;
  uint4* b4 = reinterpret_cast<uint4*>(bits);
  int64_t e0 = start[range], e1 = start[range + 1];
  e0 = e0 < 0 ? 0 : e0;
  e1 = e1 > nnz ? nnz : e1;
  // sixteen loads per thread in flight, the first batch requested before the flags are cleared (one
  // workgroup per CU: nothing else hides the latency of the stream)
  constexpr int U = 16;
  int32_t c[U];
#pragma unroll
  for (int j = 0; j < U; ++j) c[j] = e0 + threadIdx.x + j * kLdsThreads < e1 ? cols[e0 + threadIdx.x + j * kLdsThreads] : -1;
  for (int i = threadIdx.x; i < (int)(kBktCols / 16); i += kLdsThreads) b4[i] = make_uint4(0u, 0u, 0u, 0u);
  __syncthreads();
  for (int64_t base = e0; base < e1; base += U * kLdsThreads) {
#pragma unroll
    for (int j = 0; j < U; ++j) {
      const int64_t rel = (int64_t)c[j] - c0;
      if (c[j] >= 0 && rel >= 0 && rel < kBktCols) flag[rel] = 1;
    }
    const int64_t en = base + U * kLdsThreads + threadIdx.x;
#pragma unroll
    for (int j = 0; j < U; ++j) c[j] = en + j * kLdsThreads < e1 ? cols[en + j * kLdsThreads] : -1;
  }
  __syncthreads();
  // 64 flag bytes -> one word: a lane squeezes its 8 bytes into 8 bits, eight lanes make a word
  const int64_t w0 = c0 >> 6;
  const int words_here = (int)((W - w0 < kBktCols / 64) ? (W - w0) : (kBktCols / 64));
  const uint2* f8 = reinterpret_cast<const uint2*>(bits);
  for (int i = threadIdx.x; i < words_here * 8; i += kLdsThreads) {
    const uint2 t = f8[i];
    // bytes are 0 or 1: gather bit 0 of every byte
    const uint32_t lo = ((t.x & 0x01010101u) * 0x01020408u) >> 24;
    const uint32_t hi = ((t.y & 0x01010101u) * 0x01020408u) >> 24;
    uint64_t piece = (uint64_t)((lo & 0xFu) | ((hi & 0xFu) << 4)) << ((i & 7) * 8);
    // combine the eight lanes of a word (consecutive lanes)
    piece |= __shfl_xor(piece, 1, 64);
    piece |= __shfl_xor(piece, 2, 64);
    piece |= __shfl_xor(piece, 4, 64);
    if ((i & 7) == 0) {
      const int64_t wi = w0 + (i >> 3);
      const int64_t col = wi * 64;
      if (n - col < 64) piece &= (1ull << (n - col)) - 1ull;
      bm[wi] = piece;
    }
  }
}

// Membership words from the private bitmaps.  A workgroup owns 16 consecutive 64-bit words;
// thread (wi, sl) ORs the bitmaps of groups sl, sl+16, ... for word wi, LDS combines the 16
// slices.
__global__ __launch_bounds__(kThreads) void merge_kernel(const uint32_t* __restrict__ part,
                                                         int32_t groups_per_pass, int64_t W, int64_t n,
                                                         uint64_t* __restrict__ bm) {
  __shared__ uint64_t red[16][17];
  const int wi = threadIdx.x & 15, sl = threadIdx.x >> 4;
  const int64_t w = (int64_t)blockIdx.x * 16 + wi;
  uint64_t word = 0;
  if (w < W) {
    const int64_t col = w * 64;
    const int pass = (int)(col / kLdsCols);          // kLdsCols is a multiple of 64
    const int64_t idx = (col - (int64_t)pass * kLdsCols) >> 5;
    const uint32_t* __restrict__ p = part + ((size_t)pass * groups_per_pass) * kLdsWords + idx;
#pragma unroll 4
    for (int g = sl; g < groups_per_pass; g += 16) {
      const uint2 t = *reinterpret_cast<const uint2*>(p + (size_t)g * kLdsWords);
      word |= (uint64_t)t.x | ((uint64_t)t.y << 32);
    }
  }
  red[sl][wi] = word;
  __syncthreads();
  if (sl == 0 && w < W) {
#pragma unroll
    for (int j = 1; j < 16; ++j) word |= red[j][wi];
    const int64_t col = w * 64;
    if (n - col < 64) word &= (1ull << (n - col)) - 1ull;
    bm[w] = word;
  }
}

// blocksum[b] = number of set bits in the b-th tile of kWordsPerBlock words (what words_kernel
// produces on the byte-flag path)
__global__ __launch_bounds__(kThreads) void count_kernel(const uint64_t* __restrict__ bm, int64_t W,
                                                         int32_t* __restrict__ blocksum) {
  __shared__ int wsum[kThreads / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int cnt = 0;
  for (int i = threadIdx.x; i < kWordsPerBlock; i += kThreads) {
    const int64_t w = (int64_t)blockIdx.x * kWordsPerBlock + i;
    if (w < W) cnt += __popcll(bm[w]);
  }
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) cnt += __shfl_xor(cnt, d, 64);
  if (lane == 0) wsum[wave] = cnt;
  __syncthreads();
  if (threadIdx.x == 0) {
    int t = 0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) t += wsum[w];
    blocksum[blockIdx.x] = t;
  }
}

__device__ __forceinline__ int wave_inclusive_scan(int v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int t = __shfl_up(v, d, 64);
    if (lane >= d) v += t;
  }
  return v;
}

// exclusive scan over the kThreads threads of a block; returns the exclusive prefix of v and
// the block total through *total
__device__ __forceinline__ int block_exclusive_scan(int v, int* total) {
  __shared__ int wsum[kThreads / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int inc = wave_inclusive_scan(v);
  if (lane == 63) wsum[wave] = inc;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kThreads / 64; ++w) {
    const int s = wsum[w];
    if (w < wave) base += s;
    tot += s;
  }
  __syncthreads();
  *total = tot;
  return base + inc - v;
}

// Membership words from the flag bytes.  A block owns kWordsPerBlock consecutive words; each of
// its wavefronts walks its share 16 words (1024 flag bytes) per step: a lane loads 16 flags with
// one 16-byte load and squeezes them into 16 bits (flags are 0 or 1: a multiply gathers the low
// bit of every byte), four neighbouring lanes OR their quarters into one word.
__device__ __forceinline__ uint32_t squeeze8(uint64_t x) {
  return (uint32_t)(((x & 0x0101010101010101ull) * 0x0102040810204080ull) >> 56);
}

__global__ __launch_bounds__(kThreads) void words_kernel(const uint8_t* __restrict__ flag, int64_t W,
                                                         uint64_t* __restrict__ bm,
                                                         int32_t* __restrict__ blocksum) {
  __shared__ int wsum[kThreads / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  constexpr int kPerWave = kWordsPerBlock / (kThreads / 64);
  static_assert(kPerWave % 16 == 0, "a wavefront step covers 16 words");
  const int64_t w0 = (int64_t)blockIdx.x * kWordsPerBlock + (int64_t)wave * kPerWave;
  const ulonglong2* __restrict__ f16 = reinterpret_cast<const ulonglong2*>(flag);   // flag is 256-byte aligned
  int cnt = 0;
  for (int i = 0; i < kPerWave; i += 16) {
    const int64_t w = w0 + i + (lane >> 2);
    ulonglong2 v = make_ulonglong2(0ull, 0ull);
    if (w < W) v = f16[(w0 + i) * 4 + lane];
    const uint64_t quarter = (uint64_t)(squeeze8(v.x) | (squeeze8(v.y) << 8));
    cnt += __popcll(quarter);
    uint64_t word = quarter << (16 * (lane & 3));
    word |= __shfl_xor(word, 1, 64);
    word |= __shfl_xor(word, 2, 64);
    if ((lane & 3) == 0 && w < W) bm[w] = word;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) cnt += __shfl_down(cnt, o, 64);
  if (lane == 0) wsum[wave] = cnt;
  __syncthreads();
  if (threadIdx.x == 0) {
    int t = 0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) t += wsum[w];
    blocksum[blockIdx.x] = t;
  }
}

// one workgroup: in-place exclusive scan of blocksum[0..nblk), blocksum[nblk] = grand total
__global__ __launch_bounds__(kThreads) void scan_blocks_kernel(int32_t* __restrict__ blocksum,
                                                               int64_t nblk) {
  int carry = 0;
  for (int64_t base = 0; base < nblk; base += kThreads) {
    const int64_t i = base + threadIdx.x;
    const int v = (i < nblk) ? blocksum[i] : 0;
    int total;
    const int ex = block_exclusive_scan(v, &total);
    if (i < nblk) blocksum[i] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0) blocksum[nblk] = carry;
}

// A tile of kWordsPerBlock words goes through LDS so that both the loads of the words and the
// stores of the prefix counts and rank records are coalesced (thread t of step i moves element
// t + 256 i), while the scan still gives a thread eight consecutive words.
__global__ __launch_bounds__(kThreads) void prefix_kernel(const uint64_t* __restrict__ bm,
                                                          int64_t W,
                                                          const int32_t* __restrict__ blocksum,
                                                          int64_t nblk, int32_t* __restrict__ prefix,
                                                          uint4* __restrict__ rank16) {
  __shared__ uint64_t words[kWordsPerBlock];
  __shared__ int32_t pre[kWordsPerBlock];
  const int64_t tile0 = (int64_t)blockIdx.x * kWordsPerBlock;
#pragma unroll
  for (int i = 0; i < kWordsPerBlock / kThreads; ++i) {
    const int j = threadIdx.x + i * kThreads;
    words[j] = tile0 + j < W ? bm[tile0 + j] : 0ull;
  }
  __syncthreads();
  int c[8];
  int s = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    c[i] = __popcll(words[threadIdx.x * 8 + i]);
    s += c[i];
  }
  int total;
  int run = blocksum[blockIdx.x] + block_exclusive_scan(s, &total);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    pre[threadIdx.x * 8 + i] = run;
    run += c[i];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kWordsPerBlock / kThreads; ++i) {
    const int j = threadIdx.x + i * kThreads;
    if (tile0 + j < W) {
      const uint64_t word = words[j];
      const int32_t p = pre[j];
      prefix[tile0 + j] = p;
      rank16[tile0 + j] = make_uint4((uint32_t)word, (uint32_t)(word >> 32), (uint32_t)p, 0u);
    }
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) prefix[W] = blocksum[nblk];
}

__device__ __forceinline__ int rank_of(const uint64_t* __restrict__ bm,
                                       const int32_t* __restrict__ prefix, int64_t c) {
  const int64_t w = c >> 6;
  const uint64_t below = bm[w] & ((1ull << (c & 63)) - 1ull);
  return prefix[w] + __popcll(below);
}

__global__ void blkoff_kernel(const uint64_t* __restrict__ bm, const int32_t* __restrict__ prefix,
                              int64_t W, int64_t n, const int64_t* __restrict__ colblk, int32_t nb,
                              int64_t* __restrict__ blkoff) {
  for (int q = threadIdx.x; q <= nb; q += blockDim.x) {
    const int64_t c = colblk[q];
    blkoff[q] = (c >= n || (c >> 6) >= W) ? (int64_t)prefix[W] : (int64_t)rank_of(bm, prefix, c);
  }
}

// one wavefront per bitmap word
__global__ __launch_bounds__(kThreads) void emit_kernel(const uint64_t* __restrict__ bm,
                                                        const int32_t* __restrict__ prefix,
                                                        int64_t W, int64_t n,
                                                        int32_t* __restrict__ needed) {
  const int lane = threadIdx.x & 63;
  const int64_t wave0 = ((int64_t)blockIdx.x * kThreads + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * kThreads) >> 6;
  for (int64_t w = wave0; w < W; w += nwaves) {
    const uint64_t word = bm[w];
    const int64_t c = w * 64 + lane;
    const bool set = ((word >> lane) & 1ull) != 0 && c < n;
    const uint64_t mask = __ballot(set);
    const int slot = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                               __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
    if (set) needed[(int64_t)prefix[w] + slot] = (int32_t)c;
  }
}

// Sparse membership (a few needed columns per word, e.g. a rank's share of a huge graph): one
// thread per word walks the set bits; a wavefront per word would write a handful of ids with
// 64 lanes.
__global__ __launch_bounds__(kThreads) void emit_sparse_kernel(const uint64_t* __restrict__ bm,
                                                               const int32_t* __restrict__ prefix,
                                                               int64_t W, int64_t n,
                                                               int32_t* __restrict__ needed) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t w = (int64_t)blockIdx.x * kThreads + threadIdx.x; w < W; w += stride) {
    uint64_t word = bm[w];
    if (word == 0ull) continue;
    int64_t pos = prefix[w];
    const int64_t base = w * 64;
    while (word) {
      const int b = __builtin_ctzll(word);
      word &= word - 1ull;
      if (base + b < n) needed[pos++] = (int32_t)(base + b);
    }
  }
}

__device__ __forceinline__ int32_t remap_one(int32_t c, int64_t n, const uint4* __restrict__ rank16) {
  if (c < 0 || c >= n) return -1;
  const uint4 t = rank16[c >> 6];
  const uint64_t word = (uint64_t)t.x | ((uint64_t)t.y << 32);
  return (int32_t)t.z + __popcll(word & ((1ull << (c & 63)) - 1ull));
}

__global__ __launch_bounds__(kThreads) void remap_kernel(const int32_t* __restrict__ colidx,
                                                         int64_t nnz, int64_t n,
                                                         const uint4* __restrict__ rank16,
                                                         int32_t* __restrict__ compact, int aligned) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  const int64_t quads = aligned ? (nnz >> 2) : 0;
  const int4* __restrict__ c4 = reinterpret_cast<const int4*>(colidx);
  int4* __restrict__ o4 = reinterpret_cast<int4*>(compact);
  for (int64_t q = (int64_t)blockIdx.x * kThreads + threadIdx.x; q < quads; q += stride) {
    const int4 c = c4[q];
    int4 o;
    o.x = remap_one(c.x, n, rank16);
    o.y = remap_one(c.y, n, rank16);
    o.z = remap_one(c.z, n, rank16);
    o.w = remap_one(c.w, n, rank16);
    o4[q] = o;
  }
  for (int64_t e = (quads << 2) + (int64_t)blockIdx.x * kThreads + threadIdx.x; e < nnz; e += stride)
    compact[e] = remap_one(colidx[e], n, rank16);
}

// Every column is needed (N == n, e.g. a whole graph planned as one block): the position of
// column c in needed[] is c itself, so the remap is a range-checked copy (pure streaming).
__global__ __launch_bounds__(kThreads) void remap_identity_kernel(const int32_t* __restrict__ colidx,
                                                                  int64_t nnz, int64_t n,
                                                                  int32_t* __restrict__ compact,
                                                                  int aligned) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  const int64_t quads = aligned ? (nnz >> 2) : 0;
  const int4* __restrict__ c4 = reinterpret_cast<const int4*>(colidx);
  int4* __restrict__ o4 = reinterpret_cast<int4*>(compact);
  auto one = [n](int32_t c) { return (c < 0 || c >= n) ? -1 : c; };
  for (int64_t q = (int64_t)blockIdx.x * kThreads + threadIdx.x; q < quads; q += stride) {
    const int4 c = c4[q];
    o4[q] = make_int4(one(c.x), one(c.y), one(c.z), one(c.w));
  }
  for (int64_t e = (quads << 2) + (int64_t)blockIdx.x * kThreads + threadIdx.x; e < nnz; e += stride)
    compact[e] = one(colidx[e]);
}

inline unsigned grid_for(int64_t items, int64_t per_thread = 1) {
  int64_t b = ceil_div(ceil_div(items, per_thread), kThreads);
  const int64_t cap = 256 * 32;  // enough workgroups to fill 256 CUs several times over
  if (b > cap) b = cap;
  if (b < 1) b = 1;
  return (unsigned)b;
}

}  // namespace
}  // namespace sagnn

SAGNN_EXPORT int spmm_plan_workspace_bytes(int64_t m, int64_t n, int64_t nnz, int32_t nb,
                                           size_t* bytes) {
  using namespace sagnn;
  if (!bytes || m < 0 || n < 0 || nnz < 0 || nb < 1 || n > 0x7FFFFFFFll || nnz > 0x7FFFFFFFll)
    return SAGNN_EINVAL;
  *bytes = carve(nullptr, n, nb, nnz).bytes;
  return SAGNN_OK;
}

namespace sagnn {
namespace {

// ---------------------------------------------------------------------------------------------
// Small blocks (the launch-latency regime: a few thousand rows and columns): the whole plan in one
// workgroup and one launch.  Membership bits, their prefix counts and the validity flags live in
// LDS; the block boundaries come in as a kernel argument and the block offsets and error flags go
// out through one small record, so the call is one launch, one copy back and one wait instead of
// ten launches and three copies.  Same results as the general path: needed[] ascending, remap -1
// for a column outside [0, n), nothing written to needed[] / the remap when N exceeds the
// capacity or the validation fails.
constexpr int64_t kSmallMaxCols = 262144;   // 4096 membership words of 64 columns
constexpr int64_t kSmallMaxNnz = 65536;
constexpr int64_t kSmallMaxRows = 262144;
constexpr int32_t kSmallMaxBlocks = 16;
struct SmallColblk { int64_t v[kSmallMaxBlocks + 1]; };
struct SmallOut {
  int32_t err[4];
  int64_t blkoff[kSmallMaxBlocks + 1];
};
static_assert(sizeof(SmallOut) <= 256, "the record shares the 256-byte slot of the error counters");

__global__ __launch_bounds__(1024) void plan_small_kernel(const int32_t* __restrict__ rowptr,
                                                          const int32_t* __restrict__ colidx, int64_t m, int64_t n,
                                                          int64_t nnz, const SmallColblk cb, int32_t nb,
                                                          int32_t* __restrict__ needed, int64_t needed_cap,
                                                          int32_t* __restrict__ compact, int32_t validate,
                                                          SmallOut* __restrict__ out) {
  __shared__ uint64_t bm[kSmallMaxCols / 64];
  __shared__ int32_t pre[kSmallMaxCols / 64 + 1];
  __shared__ int32_t wsum[16];
  __shared__ int32_t bad[2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int W = (int)((n + 63) >> 6);
  for (int i = tid; i < W; i += 1024) bm[i] = 0ull;
  if (tid < 2) bad[tid] = 0;
  __syncthreads();
  if (validate) {
    for (int64_t r = tid; r < m; r += 1024)
      if (rowptr[r] > rowptr[r + 1]) bad[0] = 1;
    if (tid == 0 && (rowptr[0] != 0 || (int64_t)rowptr[m] != nnz)) bad[0] = 1;
  }
  uint32_t* bits = reinterpret_cast<uint32_t*>(bm);   // bit c of the 64-bit word c >> 6 = bit c & 31 of 32-bit word c >> 5
  // (eight loads in flight per thread: one workgroup has to hide the memory latency by itself)
  for (int64_t e0 = tid; e0 < nnz; e0 += 8 * 1024) {
    int32_t c8[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) c8[j] = e0 + j * 1024 < nnz ? colidx[e0 + j * 1024] : 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (e0 + j * 1024 >= nnz) continue;
      const int32_t c = c8[j];
      if (c < 0 || c >= n) {
        bad[1] = 1;
      } else {
        const uint32_t bit = 1u << (c & 31);
        if ((__hip_atomic_load(&bits[c >> 5], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) & bit) == 0)
          __hip_atomic_fetch_or(&bits[c >> 5], bit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      }
    }
  }
  __syncthreads();
  // prefix counts: thread t owns words 4t .. 4t + 3
  int cnt[4], sum = 0;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int w = 4 * tid + k;
    cnt[k] = w < W ? __popcll(bm[w]) : 0;
    sum += cnt[k];
  }
  int inc = sum;
  for (int o = 1; o < 64; o <<= 1) {
    const int t = __shfl_up(inc, o, 64);
    if (lane >= o) inc += t;
  }
  if (lane == 63) wsum[wave] = inc;
  __syncthreads();
  int before = 0, N = 0;
  for (int j = 0; j < 16; ++j) {
    if (j < wave) before += wsum[j];
    N += wsum[j];
  }
  int run = before + inc - sum;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int w = 4 * tid + k;
    if (w < W) pre[w] = run;
    run += cnt[k];
  }
  if (tid == 0) pre[W] = N;
  __syncthreads();
  auto rank = [&](int64_t c) -> int32_t {
    if (c >= n) return N;
    const int w = (int)(c >> 6);
    return pre[w] + __popcll(bm[w] & ((1ull << (c & 63)) - 1ull));
  };
  for (int q = tid; q <= nb; q += 1024) out->blkoff[q] = rank(cb.v[q]);
  if (tid < 4) out->err[tid] = tid < 2 ? bad[tid] : 0;
  if ((int64_t)N > needed_cap || (validate && (bad[0] || bad[1]))) return;   // (the same for every thread)
  for (int w = wave; w < W; w += 16) {     // one wavefront per word: lane = column, slot from the lanes below
    const uint64_t x = bm[w];
    const bool set = (x >> lane) & 1ull;
    const int slot = __popcll(x & ((1ull << lane) - 1ull));
    if (set) needed[pre[w] + slot] = w * 64 + lane;
  }
  if (compact)
    for (int64_t e0 = tid; e0 < nnz; e0 += 8 * 1024) {
      int32_t c8[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) c8[j] = e0 + j * 1024 < nnz ? colidx[e0 + j * 1024] : 0;
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (e0 + j * 1024 < nnz) compact[e0 + j * 1024] = (c8[j] < 0 || c8[j] >= n) ? -1 : rank(c8[j]);
    }
}

}  // namespace
}  // namespace sagnn

namespace sagnn {
namespace {

// host-side argument checks shared by the two planning entry points (no HIP call is made)
int plan_check_args(const int32_t* d_rowptr, const int32_t* d_colidx, int64_t m, int64_t n,
                    int64_t nnz, const int64_t* h_colblk, int32_t nb, const int32_t* d_needed,
                    int64_t needed_cap, const int64_t* h_blk_off) {
  if (m < 0 || n < 0 || nnz < 0 || nb < 1 || needed_cap < 0 || n > 0x7FFFFFFFll ||
      nnz > 0x7FFFFFFFll || m > 0x7FFFFFFFll)
    return SAGNN_EINVAL;
  if (!h_colblk || !h_blk_off || !d_rowptr) return SAGNN_EINVAL;
  if (nnz > 0 && !d_colidx) return SAGNN_EINVAL;
  if (needed_cap > 0 && !d_needed) return SAGNN_EINVAL;
  if (h_colblk[0] != 0 || h_colblk[nb] != n) return SAGNN_EFORMAT;
  for (int32_t q = 0; q < nb; ++q)
    if (h_colblk[q] > h_colblk[q + 1]) return SAGNN_EFORMAT;
  return SAGNN_OK;
}

// the planning pipeline on an already carved workspace (w.part == nullptr: byte-flag marking)
int plan_run(const int32_t* d_rowptr, const int32_t* d_colidx, int64_t m, int64_t n, int64_t nnz,
             const int64_t* h_colblk, int32_t nb, int32_t* d_needed, int64_t needed_cap,
             int64_t* h_blk_off, int32_t* d_colidx_compact, const PlanWs& w, uint32_t flags,
             hipStream_t s) {

  if ((flags & (SAGNN_PLAN_OBLIVIOUS | SAGNN_PLAN_MULTIPASS)) == 0 && n <= kSmallMaxCols && nnz <= kSmallMaxNnz && m <= kSmallMaxRows &&
      nb <= kSmallMaxBlocks) {
    // one launch, one copy back, one wait (the record lies in the slot of the error counters)
    SmallColblk cb{};
    for (int32_t q = 0; q <= nb; ++q) cb.v[q] = h_colblk[q];
    SmallOut* d_out = reinterpret_cast<SmallOut*>(w.err);
    hipLaunchKernelGGL(plan_small_kernel, dim3(1), dim3(1024), 0, s, d_rowptr, d_colidx, m, n, nnz, cb, nb, d_needed,
                       needed_cap, d_colidx_compact, (flags & SAGNN_PLAN_VALIDATE) ? 1 : 0, d_out);
    SAGNN_LAUNCH_CHECK();
    SmallOut h_out;
    SAGNN_HIP(hipMemcpyAsync(&h_out, d_out, sizeof(SmallOut), hipMemcpyDeviceToHost, s));
    SAGNN_HIP(hipStreamSynchronize(s));
    for (int32_t q = 0; q <= nb; ++q) h_blk_off[q] = h_out.blkoff[q];
    if ((flags & SAGNN_PLAN_VALIDATE) && (h_out.err[0] || h_out.err[1])) return SAGNN_EFORMAT;
    if (h_blk_off[nb] > needed_cap) return SAGNN_ECAPACITY;
    return SAGNN_OK;
  }
  SAGNN_HIP(hipMemcpyAsync(w.colblk, h_colblk, sizeof(int64_t) * (size_t)(nb + 1),
                           hipMemcpyHostToDevice, s));
  // (the bucketed marking does not use the flag bytes: only the error counters are cleared then)
  const int64_t clear16 = ((flags & SAGNN_PLAN_OBLIVIOUS) == 0 && w.bkt_cols != nullptr) ? 0 : w.W * 4;
  hipLaunchKernelGGL(clear_kernel, dim3(grid_for(clear16)), dim3(kThreads), 0, s,
                     reinterpret_cast<uint4*>(w.flag), clear16, w.err);
  SAGNN_LAUNCH_CHECK();
  if (flags & SAGNN_PLAN_VALIDATE) {
    hipLaunchKernelGGL(validate_rowptr_kernel, dim3(grid_for(m)), dim3(kThreads), 0, s, d_rowptr,
                       m, nnz, w.err);
    SAGNN_LAUNCH_CHECK();
  }
  const bool oblivious = (flags & SAGNN_PLAN_OBLIVIOUS) != 0;
  const bool bucket_mark = !oblivious && w.bkt_cols != nullptr;
  const bool lds_mark = !oblivious && !bucket_mark && w.part != nullptr;
  bool speculated = false;   // the marking pass has already written the identity remap
  if (bucket_mark) {
    const int32_t nbk = (int32_t)bucket_ranges(n);
    const size_t lds = (size_t)kBktCols;
    hipLaunchKernelGGL(bucket_count_kernel, dim3(kBktGroups), dim3(kBktThreads), 0, s, d_colidx, nnz, n, nbk, w.bkt_cnt,
                       w.err);
    SAGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(bucket_within_kernel, dim3((unsigned)nbk), dim3(kBktGroups), 0, s, w.bkt_cnt, w.bkt_start);
    SAGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(bucket_starts_kernel, dim3(1), dim3(1024), 0, s, w.bkt_start, nbk);
    SAGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(bucket_scatter_kernel, dim3(kBktGroups), dim3(kBktThreads), 0, s, d_colidx, nnz, n, nbk,
                       w.bkt_cnt, w.bkt_start, w.bkt_cols, d_colidx_compact ? w.bkt_place : (int32_t*)nullptr);
    SAGNN_LAUNCH_CHECK();
    SAGNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(mark_bucket_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(mark_bucket_kernel, dim3((unsigned)nbk), dim3(kLdsThreads), lds, s, w.bkt_cols, w.bkt_start,
                       nnz, n, w.W, w.bitmap);
    SAGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(count_kernel, dim3((unsigned)w.nblk), dim3(kThreads), 0, s, w.bitmap, w.W,
                       w.blocksum);
    SAGNN_LAUNCH_CHECK();
  } else if (lds_mark) {
    const int passes = (int)ceil_div(n, kLdsCols);
    const int groups_per_pass = kLdsGroups / passes;
    const size_t lds = sizeof(uint32_t) * (size_t)kLdsWords;
    SAGNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(mark_lds_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    // dense enough that every column is probably needed: write the identity remap on the way
    speculated = d_colidx_compact && !oblivious && nnz >= 8 * n;
    const bool al = aligned16(d_colidx) && (!speculated || aligned16(d_colidx_compact));
    hipLaunchKernelGGL(mark_lds_kernel, dim3((unsigned)(passes * groups_per_pass)), dim3(kLdsThreads),
                       lds, s, d_colidx, nnz, n, (int32_t)groups_per_pass, w.part, w.err, al ? 1 : 0,
                       speculated ? d_colidx_compact : (int32_t*)nullptr);
    SAGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(merge_kernel, dim3((unsigned)ceil_div(w.W, 16)), dim3(kThreads), 0, s, w.part,
                       (int32_t)groups_per_pass, w.W, n, w.bitmap);
    SAGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(count_kernel, dim3((unsigned)w.nblk), dim3(kThreads), 0, s, w.bitmap, w.W,
                       w.blocksum);
    SAGNN_LAUNCH_CHECK();
  } else {
    if (nnz > 0 && (!oblivious || (flags & SAGNN_PLAN_VALIDATE))) {
      hipLaunchKernelGGL(mark_kernel, dim3(grid_for(nnz, 8)), dim3(kThreads), 0, s, d_colidx, nnz,
                         n, w.flag, w.err, aligned16(d_colidx) ? 1 : 0);
      SAGNN_LAUNCH_CHECK();
    }
    if (oblivious && n > 0) {
      hipLaunchKernelGGL(fill_all_kernel, dim3(grid_for(n)), dim3(kThreads), 0, s, w.flag, n);
      SAGNN_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(words_kernel, dim3((unsigned)w.nblk), dim3(kThreads), 0, s, w.flag, w.W,
                       w.bitmap, w.blocksum);
    SAGNN_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(scan_blocks_kernel, dim3(1), dim3(kThreads), 0, s, w.blocksum, w.nblk);
  SAGNN_LAUNCH_CHECK();
  hipLaunchKernelGGL(prefix_kernel, dim3((unsigned)w.nblk), dim3(kThreads), 0, s, w.bitmap, w.W,
                     w.blocksum, w.nblk, w.prefix, w.rank16);
  SAGNN_LAUNCH_CHECK();
  hipLaunchKernelGGL(blkoff_kernel, dim3(1), dim3(kThreads), 0, s, w.bitmap, w.prefix, w.W, n,
                     w.colblk, nb, w.blkoff);
  SAGNN_LAUNCH_CHECK();

  int32_t h_err[4] = {0, 0, 0, 0};
  SAGNN_HIP(hipMemcpyAsync(h_blk_off, w.blkoff, sizeof(int64_t) * (size_t)(nb + 1),
                           hipMemcpyDeviceToHost, s));
  SAGNN_HIP(hipMemcpyAsync(h_err, w.err, sizeof(h_err), hipMemcpyDeviceToHost, s));
  SAGNN_HIP(hipStreamSynchronize(s));
  if ((flags & SAGNN_PLAN_VALIDATE) && (h_err[0] || h_err[1])) return SAGNN_EFORMAT;
  const int64_t N = h_blk_off[nb];
  if (N > needed_cap) return SAGNN_ECAPACITY;

  if (N > 0) {
    if (N * 8 < n)   // fewer than 8 needed columns per word on average
      hipLaunchKernelGGL(emit_sparse_kernel, dim3(grid_for(w.W)), dim3(kThreads), 0, s, w.bitmap, w.prefix,
                         w.W, n, d_needed);
    else
      hipLaunchKernelGGL(emit_kernel, dim3(grid_for(w.W * 64)), dim3(kThreads), 0, s, w.bitmap,
                         w.prefix, w.W, n, d_needed);
    SAGNN_LAUNCH_CHECK();
  }
  if (d_colidx_compact && nnz > 0) {
    const int al = (aligned16(d_colidx) && aligned16(d_colidx_compact)) ? 1 : 0;
    if (N == n && speculated)
      return SAGNN_OK;
    if (N == n) {
      hipLaunchKernelGGL(remap_identity_kernel, dim3(grid_for(nnz, 8)), dim3(kThreads), 0, s, d_colidx,
                         nnz, n, d_colidx_compact, al);
    } else if (bucket_mark) {
      // ranks inside the buckets (in place), then every entry fetches the rank at its place
      hipLaunchKernelGGL(remap_bucket_kernel, dim3((unsigned)bucket_ranges(n)), dim3(kLdsThreads), 0, s, w.bkt_cols,
                         w.bkt_start, nnz, n, w.W, w.rank16);
      SAGNN_LAUNCH_CHECK();
      hipLaunchKernelGGL(remap_gather_kernel, dim3(kBktGroups), dim3(kBktThreads), 0, s, w.bkt_place, w.bkt_cols, nnz,
                         d_colidx_compact);
    } else
      hipLaunchKernelGGL(remap_kernel, dim3(grid_for(nnz, 8)), dim3(kThreads), 0, s, d_colidx, nnz, n,
                         w.rank16, d_colidx_compact, al);
    SAGNN_LAUNCH_CHECK();
  }
  return SAGNN_OK;
}

}  // namespace
}  // namespace sagnn

SAGNN_EXPORT int spmm_plan_needed_rows(const int32_t* d_rowptr, const int32_t* d_colidx,
                                       int64_t m, int64_t n, int64_t nnz,
                                       const int64_t* h_colblk, int32_t nb, int32_t* d_needed,
                                       int64_t needed_cap, int64_t* h_blk_off,
                                       int32_t* d_colidx_compact, void* d_ws, size_t ws_bytes,
                                       uint32_t flags, void* stream) {
  using namespace sagnn;
  int rc = plan_check_args(d_rowptr, d_colidx, m, n, nnz, h_colblk, nb, d_needed, needed_cap, h_blk_off);
  if (rc != SAGNN_OK) return rc;
  if (!d_ws || (reinterpret_cast<uintptr_t>(d_ws) & 255u)) return SAGNN_EINVAL;
  const PlanWs w = carve(d_ws, n, nb, nnz);
  if (ws_bytes < w.bytes) return SAGNN_ECAPACITY;
  return plan_run(d_rowptr, d_colidx, m, n, nnz, h_colblk, nb, d_needed, needed_cap, h_blk_off,
                  d_colidx_compact, w, flags, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------
// Planning without a caller workspace and without any allocation: the scratch arrays (column
// flags, membership words, rank records, block sums, block boundaries, error counters) live
// in a fixed array in device memory that every GPU the library runs on holds for the life of
// the process.  The host only ever sees the array through the address hipGetSymbolAddress
// returns for the current device (the symbol's name is not a device address in host code).
namespace sagnn {
namespace {

constexpr size_t kPlanStaticBytes = 8u << 20;   // 8 MiB per GPU
constexpr int kPlanStaticMaxDevices = 64;

static __device__ __align__(256) unsigned char scratch[kPlanStaticBytes];

std::mutex g_scratch_mutex;
void* g_scratch_ptr[kPlanStaticMaxDevices] = {};

// address of `scratch` on the current device, resolved once per device
int plan_static_scratch(void** out) {
  int dev = -1;
  SAGNN_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kPlanStaticMaxDevices) return SAGNN_EINVAL;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    SAGNN_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || (reinterpret_cast<uintptr_t>(p) & 255u)) return SAGNN_EINVAL;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return SAGNN_OK;
}

}  // namespace
}  // namespace sagnn

SAGNN_EXPORT int spmm_plan_needed_rows_noalloc(const int32_t* d_rowptr, const int32_t* d_colidx,
                                               int64_t m, int64_t n, int64_t nnz,
                                               const int64_t* h_colblk, int32_t nb,
                                               int32_t* d_needed, int64_t needed_cap,
                                               int64_t* h_blk_off, int32_t* d_colidx_compact,
                                               uint32_t flags, void* stream) {
  using namespace sagnn;
  int rc = plan_check_args(d_rowptr, d_colidx, m, n, nnz, h_colblk, nb, d_needed, needed_cap, h_blk_off);
  if (rc != SAGNN_OK) return rc;
  if (n > SAGNN_PLAN_NOALLOC_MAX_COLS || nb > SAGNN_PLAN_NOALLOC_MAX_BLOCKS) return SAGNN_ECAPACITY;
  // nnz = 0 in the layout: no private LDS bitmaps, the byte-flag marking path is used
  if (carve(nullptr, n, nb, 0).bytes > kPlanStaticBytes) return SAGNN_ECAPACITY;
  void* base = nullptr;
  rc = plan_static_scratch(&base);
  if (rc != SAGNN_OK) return rc;
  const PlanWs w = carve(base, n, nb, 0);
  return plan_run(d_rowptr, d_colidx, m, n, nnz, h_colblk, nb, d_needed, needed_cap, h_blk_off,
                  d_colidx_compact, w, flags, (hipStream_t)stream);
}
