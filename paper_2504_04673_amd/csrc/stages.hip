// Column-block split of a CSR row block, the stage loop of one rank of the 1.5D algorithm
// (Sec. 4.2, Alg. 2) and the communication-volume statistics of Sec. 4.1 / Table 2.
//
// The split is a one-time set-up step (the pattern is fixed for a training run), written for
// clarity: one wavefront per row, two passes (count, scatter) around a per-block scan of the
// row counts.  Inside a row the stored order is kept, so splitting does not change the order
// in which a block product sums its terms.
#include <algorithm>

#include "common.h"

namespace sagnn {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxBlocks = 256;
constexpr int kScanTile = 2048;  // elements scanned by one workgroup

struct Bounds {
  int32_t b[kMaxBlocks + 1];
};

struct SplitWs {
  int32_t* tilesum;   // [nb][ntiles + 1]
  int64_t* nnz_off;   // [nb + 1]
  int64_t ntiles;
  size_t bytes;
};

SplitWs carve_split(void* base, int64_t m, int32_t nb) {
  SplitWs w{};
  w.ntiles = ceil_div(m + 1, kScanTile);
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char* p = base ? static_cast<char*>(base) + off : nullptr;
    off += round_up(bytes, 256);
    return p;
  };
  w.tilesum = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * (size_t)nb * (size_t)(w.ntiles + 1)));
  w.nnz_off = reinterpret_cast<int64_t*>(take(sizeof(int64_t) * (size_t)(nb + 1)));
  w.bytes = off;
  return w;
}

// block of column c: largest q with b[q] <= c, or -1 if c is outside [b[0], b[nb])
__device__ __forceinline__ int find_block(const int32_t* __restrict__ b, int nb, int32_t c) {
  if (c < b[0] || c >= b[nb]) return -1;
  int lo = 0, hi = nb;  // invariant: b[lo] <= c < b[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (b[mid] <= c) lo = mid; else hi = mid;
  }
  return lo;
}

// One wavefront per row.  Lane (q & 63) keeps the running count of block q in cnt[q >> 6].
// SCATTER = false: rowptr_blk[q*(m+1) + r] = number of entries of row r in block q.
// SCATTER = true : rowptr_blk holds the per-block row pointers; entries are written to
//                  nnz_off[q] + rowptr_blk[q*(m+1) + r] + (rank among the row's entries of q).
template <bool SCATTER>
__global__ __launch_bounds__(kThreads) void split_rows_kernel(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
    const float* __restrict__ val, int64_t m, int64_t nnz, const Bounds bnd, int nb,
    int32_t* __restrict__ rowptr_blk, const int64_t* __restrict__ nnz_off,
    int32_t* __restrict__ colidx_blk, float* __restrict__ val_blk) {
  __shared__ int32_t sb[kMaxBlocks + 1];
  for (int i = threadIdx.x; i <= nb; i += kThreads) sb[i] = bnd.b[i];
  __syncthreads();
  const int lane = threadIdx.x & 63;
  const int64_t wave0 = ((int64_t)blockIdx.x * kThreads + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * kThreads) >> 6;
  for (int64_t r = wave0; r < m; r += nwaves) {
    int64_t b = rowptr[r], e = rowptr[r + 1];
    if (b < 0) b = 0;
    if (e > nnz) e = nnz;
    int32_t cnt[kMaxBlocks / 64] = {0, 0, 0, 0};
    for (int64_t base = b; base < e; base += 64) {
      const int64_t i = base + lane;
      const bool active = i < e;
      const int32_t c = active ? colidx[i] : 0;
      const int q = active ? find_block(sb, nb, c) : -1;
      uint64_t remaining = __ballot(q >= 0);
      while (remaining) {
        const int leader = __builtin_ctzll(remaining);
        const int q0 = __shfl(q, leader, 64);
        const uint64_t mask = __ballot(q == q0);
        // running count of block q0 lives on lane q0 & 63, register q0 >> 6
        int32_t have = 0;
#pragma unroll
        for (int j = 0; j < kMaxBlocks / 64; ++j) {
          const int32_t t = __shfl(cnt[j], q0 & 63, 64);
          if (j == (q0 >> 6)) have = t;
        }
        if (SCATTER && q == q0) {
          const int rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                     __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
          const int64_t o = nnz_off[q0] + rowptr_blk[(int64_t)q0 * (m + 1) + r] + have + rank;
          if (o >= 0 && o < nnz) {   // only a malformed rowptr (overlapping rows) can fail this
            colidx_blk[o] = c - sb[q0];
            val_blk[o] = val[i];
          }
        }
        if (lane == (q0 & 63)) {
#pragma unroll
          for (int j = 0; j < kMaxBlocks / 64; ++j)
            if (j == (q0 >> 6)) cnt[j] += __popcll(mask);
        }
        remaining &= ~mask;
      }
    }
    if (!SCATTER) {
#pragma unroll
      for (int j = 0; j < kMaxBlocks / 64; ++j) {
        const int q = j * 64 + lane;
        if (q < nb) rowptr_blk[(int64_t)q * (m + 1) + r] = cnt[j];
      }
    }
  }
}

__device__ __forceinline__ int wave_incl_scan(int v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int t = __shfl_up(v, d, 64);
    if (lane >= d) v += t;
  }
  return v;
}

// exclusive scan of the workgroup's kScanTile elements (8 per thread); returns the tile total
__device__ __forceinline__ int tile_scan(int (&x)[8], int (&ex)[8]) {
  __shared__ int wsum[kThreads / 64];
  int s = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) s += x[i];
  const int inc = wave_incl_scan(s);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 63) wsum[wave] = inc;
  __syncthreads();
  int base = 0, total = 0;
#pragma unroll
  for (int w = 0; w < kThreads / 64; ++w) {
    if (w < wave) base += wsum[w];
    total += wsum[w];
  }
  __syncthreads();
  int run = base + inc - s;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    ex[i] = run;
    run += x[i];
  }
  return total;
}

// grid = (ntiles, nb).  Pass 0: tile sums.  Pass 1 (after the tile sums were scanned): in-place
// exclusive scan of the counts of rows [0, m); element m receives the block total.
template <int PASS>
__global__ __launch_bounds__(kThreads) void split_scan_kernel(int32_t* __restrict__ rowptr_blk,
                                                              int64_t m, int64_t ntiles,
                                                              int32_t* __restrict__ tilesum) {
  const int q = blockIdx.y;
  int32_t* __restrict__ a = rowptr_blk + (int64_t)q * (m + 1);
  int32_t* __restrict__ ts = tilesum + (int64_t)q * (ntiles + 1);
  const int64_t i0 = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * 8;
  int x[8], ex[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = (i0 + i < m) ? a[i0 + i] : 0;
  const int total = tile_scan(x, ex);
  if (PASS == 0) {
    if (threadIdx.x == 0) ts[blockIdx.x] = total;
  } else {
    const int off = ts[blockIdx.x];
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (i0 + i < m) a[i0 + i] = off + ex[i];
    if (i0 <= m && m < i0 + 8) a[m] = ts[ntiles];   // the thread whose range holds element m
  }
}

// one workgroup per block q: exclusive scan of its tile sums, total into ts[ntiles]
__global__ __launch_bounds__(kThreads) void split_scan_tiles_kernel(int32_t* __restrict__ tilesum,
                                                                    int64_t ntiles) {
  int32_t* __restrict__ ts = tilesum + (int64_t)blockIdx.x * (ntiles + 1);
  int carry = 0;
  for (int64_t base = 0; base < ntiles; base += kScanTile) {
    const int64_t i0 = base + (int64_t)threadIdx.x * 8;
    int x[8], ex[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = (i0 + i < ntiles) ? ts[i0 + i] : 0;
    const int total = tile_scan(x, ex);
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (i0 + i < ntiles) ts[i0 + i] = carry + ex[i];
    carry += total;
  }
  if (threadIdx.x == 0) ts[ntiles] = carry;
}

// The three scan steps in one launch for rows that fit one scan tile (m + 1 <= kScanTile): one
// workgroup per block q scans its counts in place, total into element m and into ts[1] (ts laid
// out with one tile per block, as split_offsets_kernel reads it).
__global__ __launch_bounds__(kThreads) void split_scan_small_kernel(int32_t* __restrict__ rowptr_blk, int64_t m,
                                                                    int32_t* __restrict__ tilesum) {
  int32_t* __restrict__ a = rowptr_blk + (int64_t)blockIdx.x * (m + 1);
  const int64_t i0 = (int64_t)threadIdx.x * 8;
  int x[8], ex[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = (i0 + i < m) ? a[i0 + i] : 0;
  const int total = tile_scan(x, ex);
#pragma unroll
  for (int i = 0; i < 8; ++i)
    if (i0 + i < m) a[i0 + i] = ex[i];
  if (threadIdx.x == 0) {
    a[m] = total;
    tilesum[(int64_t)blockIdx.x * 2] = 0;
    tilesum[(int64_t)blockIdx.x * 2 + 1] = total;
  }
}

// nnz_off[q] = sum of the totals of blocks < q (nb <= 256; one workgroup of 256 threads: the
// totals are fetched in parallel, the running sum is taken over LDS)
__global__ __launch_bounds__(kThreads) void split_offsets_kernel(const int32_t* __restrict__ tilesum, int64_t ntiles,
                                                                 int nb, int64_t* __restrict__ nnz_off) {
  __shared__ int32_t tot[kMaxBlocks];
  if (blockIdx.x != 0) return;
  const int q = threadIdx.x;
  tot[q] = q < nb ? tilesum[(int64_t)q * (ntiles + 1) + ntiles] : 0;
  __syncthreads();
  if (threadIdx.x != 0) return;
  int64_t run = 0;
  for (int i = 0; i < nb; ++i) {
    nnz_off[i] = run;
    run += tot[i];
  }
  nnz_off[nb] = run;
}

// ------------------------------------------------------------------------------------------
// Transpose by a stable least-significant-digit radix sort of (column, entry index) pairs.
// One pass = the same three steps as the column-block split, with tiles of kSortTile entries
// in place of rows and the 256 values of an 8-bit digit in place of the column blocks: count
// per (digit, tile), scan along the tiles of each digit, scatter with the tile-local stable
// rank.  Stability makes the entries of a transposed row come out in the order of the rows
// they came from (ascending), and keeps duplicates in their stored order.
constexpr int kSortTile = 2048;       // keys per wavefront and pass
constexpr int kSortTileSmall = 256;   // for counts small enough that 2048-key tiles would leave the chip idle

template <bool SCATTER>
__global__ __launch_bounds__(kThreads) void radix_tile_kernel(
    const uint32_t* __restrict__ keys_in, const uint32_t* __restrict__ pay_in, int64_t nnz, int shift,
    int64_t ntiles, int32_t* __restrict__ counts, const int64_t* __restrict__ digit_off,
    uint32_t* __restrict__ keys_out, uint32_t* __restrict__ pay_out, int tile) {
  const int lane = threadIdx.x & 63;
  const int64_t wave0 = ((int64_t)blockIdx.x * kThreads + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * kThreads) >> 6;
  for (int64_t t = wave0; t < ntiles; t += nwaves) {
    const int64_t b = t * tile;
    const int64_t e = b + tile < nnz ? b + tile : nnz;
    int32_t cnt[4] = {0, 0, 0, 0};
    for (int64_t base = b; base < e; base += 64) {
      const int64_t i = base + lane;
      const bool active = i < e;
      const uint32_t key = active ? keys_in[i] : 0u;
      const int q = active ? (int)((key >> shift) & 255u) : -1;
      uint64_t remaining = __ballot(q >= 0);
      while (remaining) {
        const int leader = __builtin_ctzll(remaining);
        const int q0 = __shfl(q, leader, 64);
        const uint64_t mask = __ballot(q == q0);
        int32_t have = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int32_t v = __shfl(cnt[j], q0 & 63, 64);
          if (j == (q0 >> 6)) have = v;
        }
        if (SCATTER && q == q0) {
          const int rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                     __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
          const int64_t o = digit_off[q0] + counts[(int64_t)q0 * (ntiles + 1) + t] + have + rank;
          if (o >= 0 && o < nnz) {
            keys_out[o] = key;
            pay_out[o] = pay_in ? pay_in[i] : (uint32_t)i;
          }
        }
        if (lane == (q0 & 63)) {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (j == (q0 >> 6)) cnt[j] += __popcll(mask);
        }
        remaining &= ~mask;
      }
    }
    if (!SCATTER) {
#pragma unroll
      for (int j = 0; j < 4; ++j) counts[(int64_t)(j * 64 + lane) * (ntiles + 1) + t] = cnt[j];
    }
  }
}

// err[0] = 1 if some column index is outside [0, n)
__global__ __launch_bounds__(kThreads) void transpose_check_kernel(const int32_t* __restrict__ colidx,
                                                                   int64_t nnz, int64_t n,
                                                                   int32_t* __restrict__ err) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nnz; i += stride)
    if (colidx[i] < 0 || colidx[i] >= n) err[0] = 1;
}

// rowptr_t[c] = number of sorted keys below c (lower bound), c in [0, n]
__global__ __launch_bounds__(kThreads) void transpose_rowptr_kernel(const uint32_t* __restrict__ keys,
                                                                    int64_t nnz, int64_t n,
                                                                    int32_t* __restrict__ rowptr_t) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t c = (int64_t)blockIdx.x * kThreads + threadIdx.x; c <= n; c += stride) {
    int64_t lo = 0, hi = nnz;
    while (lo < hi) {
      const int64_t mid = (lo + hi) >> 1;
      if ((int64_t)keys[mid] < c) lo = mid + 1; else hi = mid;
    }
    rowptr_t[c] = (int32_t)lo;
  }
}

// entry i of the transpose is entry perm[i] of A: its column there is A's row of that entry
__global__ __launch_bounds__(kThreads) void transpose_gather_kernel(
    const int32_t* __restrict__ rowptr, const float* __restrict__ val, int64_t m, int64_t nnz,
    const uint32_t* __restrict__ perm, int32_t* __restrict__ colidx_t, float* __restrict__ val_t) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nnz; i += stride) {
    const int64_t e = perm[i];
    int64_t lo = 0, hi = m;            // largest r with rowptr[r] <= e
    while (hi - lo > 1) {
      const int64_t mid = (lo + hi) >> 1;
      if ((int64_t)rowptr[mid] <= e) lo = mid; else hi = mid;
    }
    colidx_t[i] = (int32_t)lo;
    val_t[i] = e < nnz ? val[e] : 0.f;
  }
}

unsigned wave_grid(int64_t rows) {
  int64_t b = ceil_div(rows, kThreads / 64);
  if (b > 256 * 64) b = 256 * 64;
  if (b < 1) b = 1;
  return (unsigned)b;
}

}  // namespace

namespace {
// keys per wavefront: small tiles while they still fit the one-launch scan (at most kScanTile - 1 tiles)
inline int radix_tile(int64_t n) {
  return n <= (int64_t)kSortTileSmall * (kScanTile - 1) ? kSortTileSmall : kSortTile;
}
}  // namespace

RadixWs carve_radix(void* base, int64_t n) {
  RadixWs w{};
  const int64_t cap = n > 0 ? n : 1;
  w.ntiles = ceil_div(cap, radix_tile(cap));
  w.nscan = ceil_div(w.ntiles + 1, kScanTile);
  // sized for the count that needs the most tiles among all counts <= cap
  const int64_t max_tiles = std::max(w.ntiles, std::min<int64_t>(ceil_div(cap, kSortTileSmall), kScanTile - 1));
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char* p = base ? static_cast<char*>(base) + off : nullptr;
    off += round_up(bytes, 256);
    return p;
  };
  for (int i = 0; i < 2; ++i) {
    w.keys[i] = reinterpret_cast<uint32_t*>(take(sizeof(uint32_t) * (size_t)cap));
    w.pay[i] = reinterpret_cast<uint32_t*>(take(sizeof(uint32_t) * (size_t)cap));
  }
  w.counts = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * 256 * (size_t)(max_tiles + 1)));
  w.tilesum = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * 256 * (size_t)(w.nscan + 1)));
  w.digit_off = reinterpret_cast<int64_t*>(take(sizeof(int64_t) * 257));
  w.cap = cap;
  w.bytes = off;
  return w;
}

int radix_sort_pairs(const uint32_t* keys_in, const uint32_t* pay_in, int64_t n, int bits, const RadixWs& w0,
                     hipStream_t s, int* result) {
  RadixWs w = w0;
  if (n < 0 || n > w0.cap || bits < 1 || bits > 32) return SAGNN_EINVAL;
  const int tile = radix_tile(n > 0 ? n : 1);
  w.ntiles = ceil_div(n > 0 ? n : 1, tile);          // the workspace may have been carved for more
  w.nscan = ceil_div(w.ntiles + 1, kScanTile);
  const int passes = (bits + 7) / 8;
  const dim3 sgrid((unsigned)w.nscan, 256u);
  for (int pass = 0; pass < passes; ++pass) {
    const uint32_t* kin = pass == 0 ? keys_in : w.keys[(pass - 1) & 1];
    const uint32_t* pin = pass == 0 ? pay_in : w.pay[(pass - 1) & 1];
    hipLaunchKernelGGL(radix_tile_kernel<false>, dim3(wave_grid(w.ntiles)), dim3(kThreads), 0, s, kin, pin, n,
                       pass * 8, w.ntiles, w.counts, (const int64_t*)nullptr, (uint32_t*)nullptr,
                       (uint32_t*)nullptr, tile);
    SAGNN_LAUNCH_CHECK();
    if (w.ntiles + 1 <= kScanTile) {   // nscan == 1: the three scan steps as one launch
      hipLaunchKernelGGL(split_scan_small_kernel, dim3(256), dim3(kThreads), 0, s, w.counts, w.ntiles, w.tilesum);
      SAGNN_LAUNCH_CHECK();
    } else {
      hipLaunchKernelGGL(split_scan_kernel<0>, sgrid, dim3(kThreads), 0, s, w.counts, w.ntiles, w.nscan, w.tilesum);
      SAGNN_LAUNCH_CHECK();
      hipLaunchKernelGGL(split_scan_tiles_kernel, dim3(256), dim3(kThreads), 0, s, w.tilesum, w.nscan);
      SAGNN_LAUNCH_CHECK();
      hipLaunchKernelGGL(split_scan_kernel<1>, sgrid, dim3(kThreads), 0, s, w.counts, w.ntiles, w.nscan, w.tilesum);
      SAGNN_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(split_offsets_kernel, dim3(1), dim3(kThreads), 0, s, w.tilesum, w.nscan, 256, w.digit_off);
    SAGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(radix_tile_kernel<true>, dim3(wave_grid(w.ntiles)), dim3(kThreads), 0, s, kin, pin, n,
                       pass * 8, w.ntiles, w.counts, (const int64_t*)w.digit_off, w.keys[pass & 1],
                       w.pay[pass & 1], tile);
    SAGNN_LAUNCH_CHECK();
  }
  *result = (passes - 1) & 1;
  return SAGNN_OK;
}

namespace {

struct TransposeWs {
  RadixWs r;
  int32_t* err;
  size_t bytes;
};

TransposeWs carve_transpose(void* base, int64_t nnz) {
  TransposeWs w{};
  w.r = carve_radix(base, nnz);
  w.err = reinterpret_cast<int32_t*>(base ? static_cast<char*>(base) + w.r.bytes : nullptr);
  w.bytes = w.r.bytes + 256;
  return w;
}

}  // namespace
}  // namespace sagnn

SAGNN_EXPORT int spmm_split_workspace_bytes(int64_t m, int32_t nb, size_t* bytes) {
  using namespace sagnn;
  if (!bytes || m < 0 || m > 0x7FFFFFFFll || nb < 1 || nb > kMaxBlocks) return SAGNN_EINVAL;
  *bytes = carve_split(nullptr, m, nb).bytes;
  return SAGNN_OK;
}

SAGNN_EXPORT int spmm_split_colblocks(const int32_t* d_rowptr, const int32_t* d_colidx,
                                      const float* d_val, int64_t m, int64_t nnz,
                                      const int64_t* h_bounds, int32_t nb, int32_t* d_rowptr_blk,
                                      int32_t* d_colidx_blk, float* d_val_blk, int64_t* h_nnz_off,
                                      void* d_ws, size_t ws_bytes, void* stream) {
  using namespace sagnn;
  if (m < 0 || nnz < 0 || m > 0x7FFFFFFFll || nnz > 0x7FFFFFFFll || nb < 1 || nb > kMaxBlocks)
    return SAGNN_EINVAL;
  if (!d_rowptr || !h_bounds || !d_rowptr_blk || !h_nnz_off || !d_ws) return SAGNN_EINVAL;
  if (nnz > 0 && (!d_colidx || !d_val || !d_colidx_blk || !d_val_blk)) return SAGNN_EINVAL;
  if (reinterpret_cast<uintptr_t>(d_ws) & 255u) return SAGNN_EINVAL;
  Bounds bnd{};
  for (int32_t q = 0; q <= nb; ++q) {
    if (h_bounds[q] < 0 || h_bounds[q] > 0x7FFFFFFFll) return SAGNN_EFORMAT;
    if (q > 0 && h_bounds[q] < h_bounds[q - 1]) return SAGNN_EFORMAT;
    bnd.b[q] = (int32_t)h_bounds[q];
  }
  const SplitWs w = carve_split(d_ws, m, nb);
  if (ws_bytes < w.bytes) return SAGNN_ECAPACITY;
  hipStream_t s = (hipStream_t)stream;

  hipLaunchKernelGGL(split_rows_kernel<false>, dim3(wave_grid(m)), dim3(kThreads), 0, s, d_rowptr,
                     d_colidx, d_val, m, nnz, bnd, (int)nb, d_rowptr_blk, (const int64_t*)nullptr,
                     (int32_t*)nullptr, (float*)nullptr);
  SAGNN_LAUNCH_CHECK();
  const dim3 sgrid((unsigned)w.ntiles, (unsigned)nb);
  hipLaunchKernelGGL(split_scan_kernel<0>, sgrid, dim3(kThreads), 0, s, d_rowptr_blk, m, w.ntiles,
                     w.tilesum);
  SAGNN_LAUNCH_CHECK();
  hipLaunchKernelGGL(split_scan_tiles_kernel, dim3((unsigned)nb), dim3(kThreads), 0, s, w.tilesum,
                     w.ntiles);
  SAGNN_LAUNCH_CHECK();
  hipLaunchKernelGGL(split_scan_kernel<1>, sgrid, dim3(kThreads), 0, s, d_rowptr_blk, m, w.ntiles,
                     w.tilesum);
  SAGNN_LAUNCH_CHECK();
  hipLaunchKernelGGL(split_offsets_kernel, dim3(1), dim3(kThreads), 0, s, w.tilesum, w.ntiles, (int)nb,
                     w.nnz_off);
  SAGNN_LAUNCH_CHECK();
  if (nnz > 0 && m > 0) {
    hipLaunchKernelGGL(split_rows_kernel<true>, dim3(wave_grid(m)), dim3(kThreads), 0, s, d_rowptr,
                       d_colidx, d_val, m, nnz, bnd, (int)nb, d_rowptr_blk,
                       (const int64_t*)w.nnz_off, d_colidx_blk, d_val_blk);
    SAGNN_LAUNCH_CHECK();
  }
  SAGNN_HIP(hipMemcpyAsync(h_nnz_off, w.nnz_off, sizeof(int64_t) * (size_t)(nb + 1),
                           hipMemcpyDeviceToHost, s));
  SAGNN_HIP(hipStreamSynchronize(s));
  if (h_nnz_off[nb] > nnz) return SAGNN_EFORMAT;   // rows overlap: rowptr is not a CSR row pointer
  return SAGNN_OK;
}

SAGNN_EXPORT int spmm_transpose_workspace_bytes(int64_t nnz, size_t* bytes) {
  using namespace sagnn;
  if (!bytes || nnz < 0 || nnz > 0x7FFFFFFFll) return SAGNN_EINVAL;
  *bytes = carve_transpose(nullptr, nnz).bytes;
  return SAGNN_OK;
}

SAGNN_EXPORT int spmm_csr_transpose(const int32_t* d_rowptr, const int32_t* d_colidx,
                                    const float* d_val, int64_t m, int64_t n, int64_t nnz,
                                    int32_t* d_rowptr_t, int32_t* d_colidx_t, float* d_val_t,
                                    void* d_ws, size_t ws_bytes, void* stream) {
  using namespace sagnn;
  if (m < 0 || n < 0 || nnz < 0 || m > 0x7FFFFFFFll || n > 0x7FFFFFFFll || nnz > 0x7FFFFFFFll)
    return SAGNN_EINVAL;
  if (!d_rowptr || !d_rowptr_t || !d_ws) return SAGNN_EINVAL;
  if (nnz > 0 && (!d_colidx || !d_val || !d_colidx_t || !d_val_t)) return SAGNN_EINVAL;
  if (reinterpret_cast<uintptr_t>(d_ws) & 255u) return SAGNN_EINVAL;
  const TransposeWs w = carve_transpose(d_ws, nnz);
  if (ws_bytes < w.bytes) return SAGNN_ECAPACITY;
  hipStream_t s = (hipStream_t)stream;
  auto grid = [](int64_t items) {
    int64_t b = ceil_div(items, kThreads);
    if (b > 256 * 32) b = 256 * 32;
    if (b < 1) b = 1;
    return dim3((unsigned)b);
  };
  SAGNN_HIP(hipMemsetAsync(w.err, 0, sizeof(int32_t) * 4, s));
  const uint32_t* sorted_keys = reinterpret_cast<const uint32_t*>(d_colidx);
  const uint32_t* perm = nullptr;
  if (nnz > 0) {
    hipLaunchKernelGGL(transpose_check_kernel, grid(nnz), dim3(kThreads), 0, s, d_colidx, nnz, n, w.err);
    SAGNN_LAUNCH_CHECK();
    int bits = 1;
    while (bits < 31 && (1ll << bits) < n) ++bits;
    int res = 0;
    const int rc = radix_sort_pairs(reinterpret_cast<const uint32_t*>(d_colidx), nullptr, nnz, bits, w.r, s, &res);
    if (rc != SAGNN_OK) return rc;
    sorted_keys = w.r.keys[res];
    perm = w.r.pay[res];
  }
  hipLaunchKernelGGL(transpose_rowptr_kernel, grid(n + 1), dim3(kThreads), 0, s, sorted_keys, nnz, n,
                     d_rowptr_t);
  SAGNN_LAUNCH_CHECK();
  if (nnz > 0) {
    hipLaunchKernelGGL(transpose_gather_kernel, grid(nnz), dim3(kThreads), 0, s, d_rowptr, d_val, m, nnz,
                       perm, d_colidx_t, d_val_t);
    SAGNN_LAUNCH_CHECK();
  }
  int32_t h_err[4] = {0, 0, 0, 0};
  SAGNN_HIP(hipMemcpyAsync(h_err, w.err, sizeof(h_err), hipMemcpyDeviceToHost, s));
  SAGNN_HIP(hipStreamSynchronize(s));
  if (h_err[0]) return SAGNN_EFORMAT;
  return SAGNN_OK;
}

SAGNN_EXPORT int spmm_stage_loop(const sagnn_stage* h_stages, int32_t n_stages, int64_t m,
                                 const float* d_H, int64_t n, int64_t ldh, int32_t f,
                                 float* d_T0, float* d_T1, int64_t t_cap_rows, float* d_Z,
                                 int64_t ldz, int32_t accumulate_first, void* stream_spmm,
                                 void* stream_pack) {
  using namespace sagnn;
  if (!h_stages || n_stages < 0 || m < 0 || n < 0 || f <= 0 || t_cap_rows < 0) return SAGNN_EINVAL;
  if (!d_H || !d_Z || !d_T0 || !d_T1 || d_T0 == d_T1) return SAGNN_EINVAL;
  for (int32_t k = 0; k < n_stages; ++k) {
    const sagnn_stage& st = h_stages[k];
    if (st.N < 0 || st.nnz < 0 || !st.d_rowptr) return SAGNN_EINVAL;
    if (st.N > 0 && !st.d_rows) return SAGNN_EINVAL;
    if (st.nnz > 0 && (!st.d_colidx || !st.d_val)) return SAGNN_EINVAL;
    if (st.N > t_cap_rows) return SAGNN_ECAPACITY;
  }
  hipStream_t ss = (hipStream_t)stream_spmm, sp = (hipStream_t)stream_pack;
  const bool two = ss != sp;
  // events: packed[k] (buffer k&1 holds stage k's rows), used[k] (stage k's product has read it)
  hipEvent_t ev_start = nullptr, packed[2] = {nullptr, nullptr}, used[2] = {nullptr, nullptr};
  int rc = SAGNN_OK;
  auto destroy = [&]() {
    if (ev_start) (void)hipEventDestroy(ev_start);
    for (int i = 0; i < 2; ++i) {
      if (packed[i]) (void)hipEventDestroy(packed[i]);
      if (used[i]) (void)hipEventDestroy(used[i]);
    }
  };
#define STAGE_HIP(expr)                        \
  do {                                         \
    hipError_t _e = (expr);                    \
    if (_e != hipSuccess) {                    \
      set_hip_error(_e);                       \
      destroy();                               \
      return SAGNN_EHIP;                       \
    }                                          \
  } while (0)
  if (two) {
    STAGE_HIP(hipEventCreateWithFlags(&ev_start, hipEventDisableTiming));
    for (int i = 0; i < 2; ++i) {
      STAGE_HIP(hipEventCreateWithFlags(&packed[i], hipEventDisableTiming));
      STAGE_HIP(hipEventCreateWithFlags(&used[i], hipEventDisableTiming));
    }
    STAGE_HIP(hipEventRecord(ev_start, ss));
    STAGE_HIP(hipStreamWaitEvent(sp, ev_start, 0));
  }
  bool first = true;
  for (int32_t k = 0; k < n_stages && rc == SAGNN_OK; ++k) {
    const sagnn_stage& st = h_stages[k];
    float* T = (k & 1) ? d_T1 : d_T0;
    if (two && k >= 2) STAGE_HIP(hipStreamWaitEvent(sp, used[k & 1], 0));
    rc = spmm_pack_rows(d_H, n, ldh, f, st.d_rows, st.N, T, f, sp);
    if (rc != SAGNN_OK) break;
    if (two) {
      STAGE_HIP(hipEventRecord(packed[k & 1], sp));
      STAGE_HIP(hipStreamWaitEvent(ss, packed[k & 1], 0));
    }
    rc = spmm_csr_tallskinny(st.d_rowptr, st.d_colidx, st.d_val, m, st.N, st.nnz, T, f, f, d_Z, ldz,
                             (first && !accumulate_first) ? 0 : 1, st.d_ws, st.ws_bytes, ss);
    first = false;
    if (rc != SAGNN_OK) break;
    if (two) STAGE_HIP(hipEventRecord(used[k & 1], ss));
  }
#undef STAGE_HIP
  destroy();
  return rc;
}

SAGNN_EXPORT int spmm_volume_stats(const int64_t* h_counts, int32_t P, int32_t f,
                                   int32_t elem_bytes, double* h_out) {
  if (!h_counts || !h_out || P < 1 || f < 1 || elem_bytes < 1) return SAGNN_EINVAL;
  const double row_bytes = (double)f * (double)elem_bytes;
  double total = 0.0, max_recv = 0.0, max_send = 0.0;
  int64_t cut = 0;
  for (int32_t i = 0; i < P; ++i) {
    double recv = 0.0, send = 0.0;
    for (int32_t q = 0; q < P; ++q) {
      if (q == i) continue;
      const int64_t in = h_counts[(int64_t)i * P + q];   // P(i) needs these rows of H_q
      const int64_t out = h_counts[(int64_t)q * P + i];  // P(q) needs these rows of H_i
      if (in < 0 || out < 0) return SAGNN_EINVAL;
      recv += (double)in * row_bytes;
      send += (double)out * row_bytes;
      if (in > cut) cut = in;
    }
    total += recv;
    if (recv > max_recv) max_recv = recv;
    if (send > max_send) max_send = send;
  }
  const double avg = total / (double)P;
  h_out[0] = total;
  h_out[1] = avg;
  h_out[2] = max_recv;
  h_out[3] = avg > 0.0 ? (max_recv / avg - 1.0) * 100.0 : 0.0;
  h_out[4] = max_send;
  h_out[5] = avg > 0.0 ? (max_send / avg - 1.0) * 100.0 : 0.0;
  h_out[6] = (double)cut;
  h_out[7] = (double)cut * row_bytes;
  return SAGNN_OK;
}
