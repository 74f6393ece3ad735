// Dense-tile schedule of the local SpMM (Alg. 1 / 2, `Z <- Z + SpMM(A, H)`): the part of A whose
// rows and columns both belong to high-degree vertices is dense enough that a tile of it re-uses
// every row of the dense operand many times.  That part is taken out of the matrix once, at
// preparation time (the pattern is fixed for a training run, Sec. 4.1), and multiplied by a
// kernel that stages the rows of the dense operand in LDS:
//
//   * rows of A are ranked by their number of entries, columns by the number of entries that
//     reference them (two stable radix sorts); the first KR rows / KC columns form a grid of
//     tiles of RG rows x TC columns (RG = 512 or 256 rows whose accumulators live in the
//     registers of one workgroup of 16 wavefronts, TC columns = 64 KB of dense rows);
//   * a tile is kept when it holds at least `reuse` entries per column (every staged dense row
//     is then used that many times on average); consecutive kept tiles of a row group form work
//     items of about 32 K entries; everything else stays in a "rest" CSR (same row order, rows
//     still ascending) that goes through the other schedules;
//   * the product kernel walks an item tile by tile: the next tile's dense rows are fetched into
//     registers while the current one is multiplied out of LDS, a wavefront owns RPW rows of the
//     group and adds `value x dense row` for its entries, row by row, into registers; an item's
//     row sums go to a partial buffer and a second kernel adds the partials of a row group to C
//     in a fixed order (no floating-point atomics: results are reproducible).
//
// Summation: inside a tile a row's entries (at most TC) are summed serially, the tile sums of an
// item serially (at most 128), the item sums of a group in blocks of eight.
#include <algorithm>
#include <vector>

#include "common.h"
#include "rowload.h"

namespace sagnn {
namespace {

constexpr int kT = 256;
constexpr uint32_t kTileMagic = 0x7411E501u;

struct TileHeader {   // first 256 bytes of the tile region (device copy)
  uint32_t magic;
  uint32_t pad;
  uint64_t generation;
};

inline dim3 grid_for(int64_t items, int per_block = kT) {
  int64_t b = ceil_div(items, per_block);
  if (b > 256 * 64) b = 256 * 64;
  if (b < 1) b = 1;
  return dim3((unsigned)b);
}

// ---- preparation kernels -------------------------------------------------------------------

// sort keys of the rows (descending number of entries) and a check of the row pointer
__global__ __launch_bounds__(kT) void tile_rowkeys_kernel(const int32_t* __restrict__ rowptr, int64_t m,
                                                          int64_t nnz, uint32_t* __restrict__ keys,
                                                          int32_t* __restrict__ rest_rowptr,
                                                          int32_t* __restrict__ err) {
  const int64_t stride = (int64_t)gridDim.x * kT;
  for (int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x; i < m; i += stride) {
    const int64_t b = rowptr[i], e = rowptr[i + 1];
    int64_t d = e - b;
    if (b < 0 || e < b || e > nnz || (i == 0 && b != 0) || (i == m - 1 && e != nnz)) { err[0] = 1; d = 0; }
    keys[i] = 0x7FFFFFFFu - (uint32_t)d;
    rest_rowptr[i] = (int32_t)d;   // entries that stay in the rest: all of them until a kept tile says otherwise
  }
}

__global__ __launch_bounds__(kT) void tile_colcount_kernel(const int32_t* __restrict__ colidx, int64_t nnz,
                                                           int64_t k, int32_t* __restrict__ colcnt) {
  const int64_t stride = (int64_t)gridDim.x * kT;
  for (int64_t e = (int64_t)blockIdx.x * kT + threadIdx.x; e < nnz; e += stride) {
    const uint32_t c = (uint32_t)colidx[e];
    if (c < (uint64_t)k) atomicAdd(&colcnt[c], 1);
  }
}

__global__ __launch_bounds__(kT) void tile_colkeys_kernel(const int32_t* __restrict__ colcnt, int64_t k,
                                                          uint32_t* __restrict__ keys) {
  const int64_t stride = (int64_t)gridDim.x * kT;
  for (int64_t j = (int64_t)blockIdx.x * kT + threadIdx.x; j < k; j += stride)
    keys[j] = 0x7FFFFFFFu - (uint32_t)colcnt[j];
}

// rank[id] = position of id in the sorted order for the first `top` positions; list[r] = id
// (positions past the end of the sort repeat `fill`)
__global__ __launch_bounds__(kT) void tile_rank_kernel(const uint32_t* __restrict__ order, int64_t n, int64_t top,
                                                       int64_t list_len, int32_t fill, int32_t* __restrict__ rank,
                                                       int32_t* __restrict__ list) {
  const int64_t stride = (int64_t)gridDim.x * kT;
  for (int64_t r = (int64_t)blockIdx.x * kT + threadIdx.x; r < list_len; r += stride) {
    int32_t id = fill;
    if (r < top && r < n) {
      const uint32_t o = order[r];
      if (o < (uint64_t)n) { id = (int32_t)o; rank[o] = (int32_t)r; }
    }
    list[r] = id;
  }
}

struct TileDims {
  int64_t m, k, nnz;
  int32_t rows;      // ranked rows (KRv)
  int32_t rg, tc, nc, rpw;
  int32_t row_bytes; // f * 4
};

__device__ __forceinline__ int lane_rank(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// one wavefront per ranked row: entries of the row per column chunk.
// PASS 0: added to the tile counters.  PASS 1: entries in kept tiles are written to the count
// table of their (tile, wavefront, row slot) and taken off the row's rest count.
template <int PASS>
__global__ __launch_bounds__(kT) void tile_count_kernel(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx, const int32_t* __restrict__ hubrow,
    const int32_t* __restrict__ colrank, TileDims d, int32_t* __restrict__ tilecnt,
    const int32_t* __restrict__ tileslot, const int32_t* __restrict__ ts_item, const int32_t* __restrict__ item_ts0,
    const int32_t* __restrict__ item_nch, uint16_t* __restrict__ cnt16, int32_t* __restrict__ rest_rowptr) {
  __shared__ int32_t cnt[kT / 64][1024];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  for (int64_t r = (int64_t)blockIdx.x * (kT / 64) + w; r < d.rows; r += (int64_t)gridDim.x * (kT / 64)) {
    const int32_t i = hubrow[r];
    if (i < 0) continue;
    for (int c = lane; c < d.nc; c += 64) cnt[w][c] = 0;
    int64_t b = rowptr[i], e = rowptr[i + 1];   // (pass 0 runs before the row pointer check is read back)
    b = b < 0 ? 0 : b;
    e = e > d.nnz ? d.nnz : e;
    const int64_t g = r / d.rg;
    for (int64_t q = b + lane; q < e; q += 64) {
      const uint32_t c = (uint32_t)colidx[q];
      if (c < (uint64_t)d.k) {
        const int32_t rc = colrank[c];
        if (rc >= 0) {
          const int ch = rc / d.tc;
          if (PASS == 0 || tileslot[g * d.nc + ch] >= 0) atomicAdd(&cnt[w][ch], 1);
        }
      }
    }
    int32_t taken = 0;
    const int rloc = (int)(r % d.rg), w16 = rloc & 15, rslot = rloc >> 4;
    for (int c = lane; c < d.nc; c += 64) {
      const int32_t n = cnt[w][c];
      if (n == 0) continue;
      if (PASS == 0) {
        atomicAdd(&tilecnt[g * d.nc + c], n);
      } else {
        const int32_t ts = tileslot[g * d.nc + c];
        const int32_t it = ts_item[ts], ts0 = item_ts0[it], nch = item_nch[it];
        const int64_t slot = (int64_t)ts0 * 16 + (int64_t)w16 * nch + (ts - ts0);
        cnt16[slot * d.rpw + rslot] = (uint16_t)n;
        taken += n;
      }
    }
    if (PASS == 1) {
      for (int o = 32; o > 0; o >>= 1) taken += __shfl_xor(taken, o, 64);
      if (lane == 0) rest_rowptr[i] = (int32_t)(e - b) - taken;
    }
  }
}

// entries per (tile, wavefront) and the offsets of the row slots inside it
__global__ __launch_bounds__(kT) void tile_wsum_kernel(const uint16_t* __restrict__ cnt16, int64_t n_slots, int32_t rpw,
                                                       uint16_t* __restrict__ roff16, int32_t* __restrict__ wstart) {
  const int64_t stride = (int64_t)gridDim.x * kT;
  for (int64_t sl = (int64_t)blockIdx.x * kT + threadIdx.x; sl < n_slots; sl += stride) {
    int32_t run = 0;
    for (int r = 0; r < rpw; ++r) {
      roff16[sl * rpw + r] = (uint16_t)run;
      run += cnt16[sl * rpw + r];
    }
    wstart[sl] = run;
  }
}

// exclusive scan in place of a[0..n), total to a[n]; one workgroup of 1024 threads
__global__ __launch_bounds__(1024) void tile_scan_kernel(int32_t* __restrict__ a, int64_t n) {
  __shared__ int32_t wsum[16];
  __shared__ int32_t carry_s;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  if (threadIdx.x == 0) carry_s = 0;
  __syncthreads();
  for (int64_t base = 0; base < n; base += 4096) {
    const int64_t i0 = base + (int64_t)threadIdx.x * 4;
    int32_t v[4];
    int32_t s = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      v[j] = i0 + j < n ? a[i0 + j] : 0;
      s += v[j];
    }
    int32_t inc = s;
    for (int o = 1; o < 64; o <<= 1) {
      const int32_t t = __shfl_up(inc, o, 64);
      if (lane >= o) inc += t;
    }
    if (lane == 63) wsum[w] = inc;
    __syncthreads();
    int32_t before = carry_s;
    for (int j = 0; j < w; ++j) before += wsum[j];
    int32_t run = before + inc - s;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (i0 + j < n) a[i0 + j] = run;
      run += v[j];
    }
    __syncthreads();
    if (threadIdx.x == 1023) carry_s = before + inc;
    __syncthreads();
  }
  if (threadIdx.x == 0) a[n] = carry_s;
}

// one wavefront per ranked row, batches of 64 entries in stored order: entries of kept tiles go
// to the tile streams (stored order kept inside a row of a tile), the others to the rest CSR
__global__ __launch_bounds__(kT) void tile_scatter_kernel(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx, const float* __restrict__ val,
    const int32_t* __restrict__ hubrow, const int32_t* __restrict__ colrank, TileDims d,
    const int32_t* __restrict__ tileslot, const int32_t* __restrict__ ts_item, const int32_t* __restrict__ item_ts0,
    const int32_t* __restrict__ item_nch, const uint16_t* __restrict__ roff16, const int32_t* __restrict__ wstart,
    uint2* __restrict__ ent, int64_t ent_cap, const int32_t* __restrict__ rest_rowptr, int32_t* __restrict__ rest_col,
    float* __restrict__ rest_val) {
  __shared__ int32_t cnt[kT / 64][1024];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  for (int64_t r = (int64_t)blockIdx.x * (kT / 64) + w; r < d.rows; r += (int64_t)gridDim.x * (kT / 64)) {
    const int32_t i = hubrow[r];
    if (i < 0) continue;
    for (int c = lane; c < d.nc; c += 64) cnt[w][c] = 0;
    const int64_t b = rowptr[i], e = rowptr[i + 1];
    const int64_t g = r / d.rg;
    const int rloc = (int)(r % d.rg), w16 = rloc & 15, rslot = rloc >> 4;
    int64_t restpos = rest_rowptr[i];
    const int64_t restend = rest_rowptr[i + 1];
    for (int64_t q0 = b; q0 < e; q0 += 64) {
      const int64_t q = q0 + lane;
      const bool in = q < e;
      uint32_t c = 0;
      float v = 0.f;
      int ch = -1;
      int32_t rc = -1;
      int64_t base = 0;
      if (in) {
        c = (uint32_t)colidx[q];
        v = val[q];
        if (c < (uint64_t)d.k) {
          rc = colrank[c];
          if (rc >= 0) {
            const int chq = rc / d.tc;
            const int32_t ts = tileslot[g * d.nc + chq];
            if (ts >= 0) {
              ch = chq;
              const int32_t it = ts_item[ts], ts0 = item_ts0[it], nch = item_nch[it];
              const int64_t slot = (int64_t)ts0 * 16 + (int64_t)w16 * nch + (ts - ts0);
              base = (int64_t)wstart[slot] + roff16[slot * d.rpw + rslot];
            }
          }
        }
      }
      const bool tile = ch >= 0;
      uint64_t todo = __ballot(tile);
      while (todo) {
        const int leader = __builtin_ctzll(todo);
        const int lch = __shfl(ch, leader, 64);
        const uint64_t same = __ballot(tile && ch == lch);
        const int32_t seen = cnt[w][lch];
        if (tile && ch == lch) {
          const int64_t pos = base + seen + lane_rank(same);
          if (pos >= 0 && pos < ent_cap)
            ent[pos] = make_uint2((uint32_t)(rc % d.tc) * (uint32_t)d.row_bytes, __float_as_uint(v));
        }
        if (lane == leader) cnt[w][lch] = seen + __popcll(same);
        todo &= ~same;
      }
      const uint64_t rest = __ballot(in && !tile);
      if (in && !tile) {
        const int64_t pos = restpos + lane_rank(rest);
        if (pos < restend) { rest_col[pos] = (int32_t)c; rest_val[pos] = v; }
      }
      restpos += __popcll(rest);
    }
  }
}

// rows outside the ranked set are copied to the rest CSR as they are
__global__ __launch_bounds__(kT) void tile_copy_rows_kernel(const int32_t* __restrict__ rowptr,
                                                            const int32_t* __restrict__ colidx,
                                                            const float* __restrict__ val, int64_t m,
                                                            const int32_t* __restrict__ rowrank,
                                                            const int32_t* __restrict__ rest_rowptr,
                                                            int32_t* __restrict__ rest_col, float* __restrict__ rest_val) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  for (int64_t i = (int64_t)blockIdx.x * (kT / 64) + w; i < m; i += (int64_t)gridDim.x * (kT / 64)) {
    if (rowrank[i] >= 0) continue;
    const int64_t b = rowptr[i], e = rowptr[i + 1], o = rest_rowptr[i], oe = rest_rowptr[i + 1];
    for (int64_t q = lane; q < e - b && o + q < oe; q += 64) {
      rest_col[o + q] = colidx[b + q];
      rest_val[o + q] = val[b + q];
    }
  }
}

// ---- product ---------------------------------------------------------------------------------

struct TileArgs {
  const TileHeader* hdr;
  uint64_t generation;
  const int32_t *item_ts0, *item_nch, *ts_chunk, *hubcol, *wstart;
  const uint16_t* cnt16;
  const uint2* ent;
  float* partial;
  const float* B;
  int64_t ldb;
  uint32_t kmax;
  int32_t ent_cap;   // entries the array holds (>= 1)
};

constexpr int kTileWaves = 16;
constexpr int kTileBuf = 65536;   // bytes of dense rows per tile (TC x f x 4)

template <int FPL, int RPW>
__global__ __launch_bounds__(kTileWaves * 64) void tile_spmm_kernel(const TileArgs a) {
  using vec = typename Vec<FPL>::T;
  extern __shared__ __align__(16) char smem[];   // two tile buffers, then the wavefronts' entry rings
  constexpr int kRowBytes = 256 * FPL;            // f * 4
  constexpr int kTC = kTileBuf / kRowBytes;       // columns per tile
  constexpr int kLanesPerRow = kRowBytes / 16;    // lanes that move one dense row, 16 bytes each
  constexpr int kRowsPerLoad = 64 / kLanesPerRow;
  constexpr int kRowsPerWave = kTC / kTileWaves;
  constexpr int kLoads = kRowsPerWave / kRowsPerLoad;   // 4 for every width
  if (a.hdr->magic != kTileMagic || a.hdr->generation != a.generation) return;
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int it = blockIdx.x;
  // (locals, so that the lambdas below do not make the compiler copy the argument struct to scratch)
  const uint2* __restrict__ ent = a.ent;
  const float* __restrict__ Bp = a.B;
  const int32_t* __restrict__ hubcol = a.hubcol;
  const int32_t* __restrict__ ts_chunk = a.ts_chunk;
  const uint16_t* __restrict__ cnt16 = a.cnt16;
  const int64_t ldb = a.ldb;
  const uint32_t kmax = a.kmax;
  const int ts0 = a.item_ts0[it], nch = a.item_nch[it];
  const int64_t slot0 = (int64_t)ts0 * 16 + (int64_t)w * nch;

  vec acc[RPW];
#pragma unroll
  for (int r = 0; r < RPW; ++r) acc[r] = 0.f;

  // This wavefront's entries: one run over all tiles of the item.  Batch k (64 entries, one per
  // lane) is in the registers `cur` and handed out by lane reads; batch k+1 waits in the
  // wavefront's slice of LDS, batch k+2 is on its way from memory into `stg` (two batches of
  // prefetch distance: the stream is read once, straight from HBM).  Reads past the end of the
  // stream stay inside the entry array.
  const int32_t ent_last = a.ent_cap - 1;
  auto load_batch = [&](int32_t p) {
    const int32_t q = p + lane;
    return ent[q < ent_last ? q : ent_last];
  };
  uint2* ring = reinterpret_cast<uint2*>(smem + 2 * kTileBuf) + w * 128 + lane;   // two slots of 64 entries
  int32_t pos = __builtin_amdgcn_readfirstlane(a.wstart[slot0]);
  uint2 cur = load_batch(pos);
  ring[64] = load_batch(pos + 64);          // batch 1 -> slot 1
  uint2 stg = load_batch(pos + 128);        // batch 2
  int idx = 0, batch = 0;
  constexpr uint32_t kOffMask = (uint32_t)(kTileBuf - kRowBytes);
  auto fetch = [&](uint32_t& c, float& v) {
    c = (uint32_t)__builtin_amdgcn_readlane((int)cur.x, idx) & kOffMask;
    v = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)cur.y, idx));
    if (++idx == 64) {
      idx = 0;
      ++batch;                               // now handing out batch `batch`, which is in slot batch & 1
      ring[((batch + 1) & 1) * 64] = stg;    // batch + 1 -> the slot batch - 1 has left
      stg = load_batch(pos + (batch + 2) * 64);
      cur = ring[(batch & 1) * 64];
    }
  };

  // dense rows of a tile: lane's piece of load q
  const int sub = lane / kLanesPerRow, piece = lane % kLanesPerRow;
  struct Stage { float4 v0, v1, v2, v3; };
  static_assert(kLoads == 4, "four 16-byte loads per lane and tile");
  auto tile_row = [&](int q) { return w * kRowsPerWave + q * kRowsPerLoad + sub; };
  auto fetch_tile = [&](int ci) {
    const int32_t ch = ts_chunk[ts0 + ci];
    const int32_t* hc = hubcol + (int64_t)ch * kTC;
    auto row_of = [&](int q) {
      uint32_t col = (uint32_t)hc[tile_row(q)];
      col = col > kmax ? kmax : col;
      return *reinterpret_cast<const float4*>(Bp + (int64_t)col * ldb + piece * 4);
    };
    Stage st;
    st.v0 = row_of(0); st.v1 = row_of(1); st.v2 = row_of(2); st.v3 = row_of(3);
    return st;
  };
  auto store_tile = [&](int bufi, const Stage& st) {
    char* dst = smem + bufi * kTileBuf + piece * 16;
    *reinterpret_cast<float4*>(dst + tile_row(0) * kRowBytes) = st.v0;
    *reinterpret_cast<float4*>(dst + tile_row(1) * kRowBytes) = st.v1;
    *reinterpret_cast<float4*>(dst + tile_row(2) * kRowBytes) = st.v2;
    *reinterpret_cast<float4*>(dst + tile_row(3) * kRowBytes) = st.v3;
  };
  Stage st = fetch_tile(0);
  store_tile(0, st);
  __syncthreads();

  for (int ci = 0; ci < nch; ++ci) {
    if (ci + 1 < nch) st = fetch_tile(ci + 1);
    typedef uint32_t cntvec __attribute__((ext_vector_type(RPW / 2), aligned(4)));
    const cntvec cw = *reinterpret_cast<const cntvec*>(cnt16 + (slot0 + ci) * RPW);
    const char* buf = smem + (ci & 1) * kTileBuf + lane * (FPL * 4);
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
      int n = (int)((cw[r >> 1] >> ((r & 1) * 16)) & 0xFFFFu);
      if (n > 0) {
        vec t0 = 0.f, t1 = 0.f;
        auto rd = [&](uint32_t c) { return *reinterpret_cast<const vec*>(buf + c); };
        while (n >= 4) {
          uint32_t c0, c1, c2, c3;
          float v0, v1, v2, v3;
          fetch(c0, v0); fetch(c1, v1); fetch(c2, v2); fetch(c3, v3);
          const vec b0 = rd(c0), b1 = rd(c1), b2 = rd(c2), b3 = rd(c3);
          t0 += v0 * b0;
          t1 += v1 * b1;
          t0 += v2 * b2;
          t1 += v3 * b3;
          n -= 4;
        }
        if (n & 2) {
          uint32_t c0, c1;
          float v0, v1;
          fetch(c0, v0); fetch(c1, v1);
          const vec b0 = rd(c0), b1 = rd(c1);
          t0 += v0 * b0;
          t1 += v1 * b1;
        }
        if (n & 1) {
          uint32_t c0;
          float v0;
          fetch(c0, v0);
          t0 += v0 * rd(c0);
        }
        acc[r] += t0 + t1;
      }
    }
    if (ci + 1 < nch) store_tile((ci + 1) & 1, st);
    __syncthreads();
  }
  float* out = a.partial + (int64_t)it * (kTileWaves * RPW) * (64 * FPL) + lane * FPL;
#pragma unroll
  for (int r = 0; r < RPW; ++r)
    *reinterpret_cast<vec*>(out + (int64_t)(w + 16 * r) * (64 * FPL)) = acc[r];
}

// C[row] += sum of the row's partial sums over the items of its group (blocks of eight, fixed order)
template <int FPL>
__global__ __launch_bounds__(kT) void tile_combine_kernel(const TileHeader* __restrict__ hdr, uint64_t generation,
                                                          const int32_t* __restrict__ hubrow,
                                                          const int32_t* __restrict__ group_item0,
                                                          const float* __restrict__ partial, int32_t rows, int32_t rg,
                                                          int64_t m, float* __restrict__ C, int64_t ldc) {
  using vec = typename Vec<FPL>::T;
  if (hdr->magic != kTileMagic || hdr->generation != generation) return;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int64_t r = (int64_t)blockIdx.x * (kT / 64) + w;
  if (r >= rows) return;
  const int32_t row = hubrow[r];
  if (row < 0 || row >= m) return;
  const int g = (int)(r / rg), rloc = (int)(r % rg);
  const int32_t i0 = group_item0[g], i1 = group_item0[g + 1];
  if (i1 <= i0) return;
  vec total = 0.f;
  for (int32_t ib = i0; ib < i1; ib += 8) {
    vec blk = 0.f;
    const int32_t ie = ib + 8 < i1 ? ib + 8 : i1;
    for (int32_t it = ib; it < ie; ++it)
      blk += *reinterpret_cast<const vec*>(partial + ((int64_t)it * rg + rloc) * (64 * FPL) + lane * FPL);
    total += blk;
  }
  vec* dst = reinterpret_cast<vec*>(C + (int64_t)row * ldc + lane * FPL);
  *dst = *dst + total;
}

}  // namespace

// ---- host side -------------------------------------------------------------------------------

bool tile_geom(int32_t f, TileGeom* g) {
  if (f != 64 && f != 128 && f != 256) return false;
  g->fpl = f / 64;
  g->rpw = f == 256 ? 16 : 32;
  g->rg = 16 * g->rpw;
  g->tc = kTileBuf / (f * 4);
  return true;
}

TileWsLayout tile_ws_layout(int64_t m, int64_t k, int64_t nnz, int32_t f) {
  TileWsLayout L{};
  TileGeom g{};
  if (!tile_geom(f, &g)) return L;
  L.kr = (int64_t)std::min<int64_t>(kTileMaxRows, (int64_t)round_up((size_t)std::max<int64_t>(m, 1), g.rg));
  L.kc = (int64_t)std::min<int64_t>(kTileMaxCols, (int64_t)round_up((size_t)std::max<int64_t>(k, 1), g.tc));
  L.ng = L.kr / g.rg;
  L.nc = L.kc / g.tc;
  L.max_ts = std::min<int64_t>(L.ng * L.nc, nnz / 256 + 1);
  L.max_items = nnz / kTileItemEntries + L.ng + 1;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += round_up(bytes, 256); return o; };
  L.header = take(256);
  L.rowrank = take(4 * (size_t)(m + 1));
  L.colrank = take(4 * (size_t)(k + 1));
  L.hubrow = take(4 * (size_t)L.kr);
  L.hubcol = take(4 * (size_t)L.kc);
  L.tilecnt = take(4 * (size_t)(L.ng * L.nc));
  L.tileslot = take(4 * (size_t)(L.ng * L.nc));
  L.ts_chunk = take(4 * (size_t)L.max_ts);
  L.ts_item = take(4 * (size_t)L.max_ts);
  L.item_g = take(4 * (size_t)L.max_items);
  L.item_ts0 = take(4 * (size_t)L.max_items);
  L.item_nch = take(4 * (size_t)L.max_items);
  L.group_item0 = take(4 * (size_t)(L.ng + 1));
  L.cnt16 = take(2 * (size_t)L.max_ts * 16 * g.rpw);
  L.roff16 = take(2 * (size_t)L.max_ts * 16 * g.rpw);
  L.wstart = take(4 * (size_t)(L.max_ts * 16 + 1));
  L.ent = take(8 * (size_t)std::max<int64_t>(nnz, 1));
  L.partial = take(4 * (size_t)L.max_items * g.rg * f);
  L.rest_rowptr = take(4 * (size_t)(m + 1));
  L.rest_col = take(4 * (size_t)std::max<int64_t>(nnz, 1));
  L.rest_val = take(4 * (size_t)std::max<int64_t>(nnz, 1));
  L.keys = take(4 * (size_t)std::max<int64_t>(std::max(m, k), 1));
  L.colcnt = take(4 * (size_t)(k + 1));
  L.err = take(256);
  L.radix = off;
  off += round_up(carve_radix(nullptr, std::max<int64_t>(std::max(m, k), 1)).bytes, 256);
  L.total = off;
  return L;
}

// Splits A into kept tiles + rest.  Returns SAGNN_OK with out->n_ts == 0 when no tile is dense
// enough (nothing was written that a later product would read).  Synchronises the stream.
int tile_prepare(const int32_t* d_rowptr, const int32_t* d_colidx, const float* d_val, int64_t m, int64_t k,
                 int64_t nnz, int32_t f, char* base, const TileWsLayout& L, int32_t reuse_x10, uint64_t generation,
                 hipStream_t s, TilePlan* out) {
  TileGeom g{};
  *out = TilePlan{};
  if (!tile_geom(f, &g) || L.total == 0) return SAGNN_EINVAL;
  if (m <= 0 || k <= 0 || nnz <= 0) return SAGNN_OK;
  auto P32 = [&](size_t o) { return reinterpret_cast<int32_t*>(base + o); };
  uint32_t* keys = reinterpret_cast<uint32_t*>(base + L.keys);
  int32_t* err = P32(L.err);
  const RadixWs rw = carve_radix(base + L.radix, std::max(m, k));
  const int64_t rows = std::min<int64_t>(L.kr, m), cols = std::min<int64_t>(L.kc, k);

  SAGNN_HIP(hipMemsetAsync(err, 0, 256, s));
  SAGNN_HIP(hipMemsetAsync(P32(L.colcnt), 0, 4 * (size_t)(k + 1), s));
  SAGNN_HIP(hipMemsetAsync(P32(L.rowrank), 0xFF, 4 * (size_t)(m + 1), s));
  SAGNN_HIP(hipMemsetAsync(P32(L.colrank), 0xFF, 4 * (size_t)(k + 1), s));
  SAGNN_HIP(hipMemsetAsync(P32(L.tilecnt), 0, 4 * (size_t)(L.ng * L.nc), s));
  hipLaunchKernelGGL(tile_rowkeys_kernel, grid_for(m), dim3(kT), 0, s, d_rowptr, m, nnz, keys, P32(L.rest_rowptr), err);
  SAGNN_LAUNCH_CHECK();
  int res = 0;
  int rc = radix_sort_pairs(keys, nullptr, m, 31, rw, s, &res);
  if (rc != SAGNN_OK) return rc;
  hipLaunchKernelGGL(tile_rank_kernel, grid_for(L.kr), dim3(kT), 0, s, rw.pay[res], m, rows, L.kr, (int32_t)-1,
                     P32(L.rowrank), P32(L.hubrow));
  SAGNN_LAUNCH_CHECK();
  hipLaunchKernelGGL(tile_colcount_kernel, grid_for(nnz), dim3(kT), 0, s, d_colidx, nnz, k, P32(L.colcnt));
  SAGNN_LAUNCH_CHECK();
  hipLaunchKernelGGL(tile_colkeys_kernel, grid_for(k), dim3(kT), 0, s, P32(L.colcnt), k, keys);
  SAGNN_LAUNCH_CHECK();
  rc = radix_sort_pairs(keys, nullptr, k, 31, rw, s, &res);
  if (rc != SAGNN_OK) return rc;
  hipLaunchKernelGGL(tile_rank_kernel, grid_for(L.kc), dim3(kT), 0, s, rw.pay[res], k, cols, L.kc, (int32_t)0,
                     P32(L.colrank), P32(L.hubcol));
  SAGNN_LAUNCH_CHECK();

  TileDims d{};
  d.m = m; d.k = k; d.nnz = nnz;
  d.rows = (int32_t)rows; d.rg = g.rg; d.tc = g.tc; d.nc = (int32_t)L.nc; d.rpw = g.rpw; d.row_bytes = f * 4;
  const dim3 row_grid = grid_for(rows, kT / 64);
  hipLaunchKernelGGL(tile_count_kernel<0>, row_grid, dim3(kT), 0, s, d_rowptr, d_colidx, P32(L.hubrow),
                     P32(L.colrank), d, P32(L.tilecnt), nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
  SAGNN_LAUNCH_CHECK();
  std::vector<int32_t> tilecnt((size_t)(L.ng * L.nc));
  int32_t h_err[4] = {0, 0, 0, 0};
  SAGNN_HIP(hipMemcpyAsync(tilecnt.data(), P32(L.tilecnt), 4 * tilecnt.size(), hipMemcpyDeviceToHost, s));
  SAGNN_HIP(hipMemcpyAsync(h_err, err, sizeof(h_err), hipMemcpyDeviceToHost, s));
  SAGNN_HIP(hipStreamSynchronize(s));
  if (h_err[0]) return SAGNN_OK;   // not a CSR row pointer: the other schedules clamp everything; no tiles

  // selection and work items (host: one counter per tile)
  const int64_t thr = std::max<int64_t>(256, (int64_t)(reuse_x10 > 0 ? reuse_x10 : 25) * g.tc / 10);
  std::vector<int32_t> tileslot(tilecnt.size(), -1), ts_chunk, ts_item, item_g, item_ts0, item_nch,
      group_item0((size_t)L.ng + 1, 0);
  int64_t entries = 0;
  for (int64_t gi = 0; gi < L.ng; ++gi) {
    group_item0[gi] = (int32_t)item_g.size();
    int64_t in_item = 0;
    bool open = false;
    for (int64_t c = 0; c < L.nc; ++c) {
      const int64_t n = tilecnt[gi * L.nc + c];
      if (n < thr) continue;
      if ((int64_t)ts_chunk.size() >= L.max_ts) break;
      if (!open || in_item >= kTileItemEntries || item_nch.back() >= 128) {
        if ((int64_t)item_g.size() >= L.max_items) break;
        item_g.push_back((int32_t)gi);
        item_ts0.push_back((int32_t)ts_chunk.size());
        item_nch.push_back(0);
        in_item = 0;
        open = true;
      }
      tileslot[gi * L.nc + c] = (int32_t)ts_chunk.size();
      ts_item.push_back((int32_t)item_g.size() - 1);
      ts_chunk.push_back((int32_t)c);
      item_nch.back() += 1;
      in_item += n;
      entries += n;
    }
  }
  group_item0[L.ng] = (int32_t)item_g.size();
  const int64_t n_ts = (int64_t)ts_chunk.size(), n_items = (int64_t)item_g.size();
  if (n_ts == 0) return SAGNN_OK;

  auto up = [&](size_t o, const std::vector<int32_t>& v) -> hipError_t {
    return hipMemcpyAsync(base + o, v.data(), 4 * v.size(), hipMemcpyHostToDevice, s);
  };
  SAGNN_HIP(up(L.tileslot, tileslot));
  SAGNN_HIP(up(L.ts_chunk, ts_chunk));
  SAGNN_HIP(up(L.ts_item, ts_item));
  SAGNN_HIP(up(L.item_g, item_g));
  SAGNN_HIP(up(L.item_ts0, item_ts0));
  SAGNN_HIP(up(L.item_nch, item_nch));
  SAGNN_HIP(up(L.group_item0, group_item0));
  const int64_t n_slots = n_ts * 16;
  uint16_t* cnt16 = reinterpret_cast<uint16_t*>(base + L.cnt16);
  uint16_t* roff16 = reinterpret_cast<uint16_t*>(base + L.roff16);
  SAGNN_HIP(hipMemsetAsync(cnt16, 0, 2 * (size_t)n_slots * g.rpw, s));
  hipLaunchKernelGGL(tile_count_kernel<1>, row_grid, dim3(kT), 0, s, d_rowptr, d_colidx, P32(L.hubrow),
                     P32(L.colrank), d, P32(L.tilecnt), P32(L.tileslot), P32(L.ts_item), P32(L.item_ts0),
                     P32(L.item_nch), cnt16, P32(L.rest_rowptr));
  SAGNN_LAUNCH_CHECK();
  hipLaunchKernelGGL(tile_wsum_kernel, grid_for(n_slots), dim3(kT), 0, s, cnt16, n_slots, (int32_t)g.rpw, roff16,
                     P32(L.wstart));
  SAGNN_LAUNCH_CHECK();
  hipLaunchKernelGGL(tile_scan_kernel, dim3(1), dim3(1024), 0, s, P32(L.wstart), n_slots);
  SAGNN_LAUNCH_CHECK();
  hipLaunchKernelGGL(tile_scan_kernel, dim3(1), dim3(1024), 0, s, P32(L.rest_rowptr), m);
  SAGNN_LAUNCH_CHECK();
  hipLaunchKernelGGL(tile_scatter_kernel, row_grid, dim3(kT), 0, s, d_rowptr, d_colidx, d_val, P32(L.hubrow),
                     P32(L.colrank), d, P32(L.tileslot), P32(L.ts_item), P32(L.item_ts0), P32(L.item_nch), roff16,
                     P32(L.wstart), reinterpret_cast<uint2*>(base + L.ent), nnz, P32(L.rest_rowptr), P32(L.rest_col),
                     reinterpret_cast<float*>(base + L.rest_val));
  SAGNN_LAUNCH_CHECK();
  hipLaunchKernelGGL(tile_copy_rows_kernel, grid_for(m, kT / 64), dim3(kT), 0, s, d_rowptr, d_colidx, d_val, m,
                     P32(L.rowrank), P32(L.rest_rowptr), P32(L.rest_col), reinterpret_cast<float*>(base + L.rest_val));
  SAGNN_LAUNCH_CHECK();
  TileHeader h{};
  h.magic = kTileMagic;
  h.generation = generation;
  SAGNN_HIP(hipMemcpyAsync(base + L.header, &h, sizeof(h), hipMemcpyHostToDevice, s));
  int32_t totals[2] = {0, 0};
  SAGNN_HIP(hipMemcpyAsync(&totals[0], P32(L.wstart) + n_slots, 4, hipMemcpyDeviceToHost, s));
  SAGNN_HIP(hipMemcpyAsync(&totals[1], P32(L.rest_rowptr) + m, 4, hipMemcpyDeviceToHost, s));
  SAGNN_HIP(hipStreamSynchronize(s));
  if (totals[0] != entries || (int64_t)totals[0] + totals[1] != nnz) return SAGNN_OK;   // inconsistent input: no tiles
  out->n_ts = n_ts;
  out->n_items = n_items;
  out->entries = entries;
  out->rest_nnz = totals[1];
  out->rows = rows;
  return SAGNN_OK;
}

int tile_launch(const TilePlan& p, uint64_t generation, char* base, const TileWsLayout& L, const float* B,
                int64_t ldb, uint32_t kmax, int32_t f, int64_t m, float* C, int64_t ldc, hipStream_t s) {
  TileGeom g{};
  if (!tile_geom(f, &g) || p.n_items <= 0) return SAGNN_EINVAL;
  auto P32 = [&](size_t o) { return reinterpret_cast<const int32_t*>(base + o); };
  TileArgs a{};
  a.hdr = reinterpret_cast<const TileHeader*>(base + L.header);
  a.generation = generation;
  a.item_ts0 = P32(L.item_ts0); a.item_nch = P32(L.item_nch);
  a.ts_chunk = P32(L.ts_chunk); a.hubcol = P32(L.hubcol); a.wstart = P32(L.wstart);
  a.cnt16 = reinterpret_cast<const uint16_t*>(base + L.cnt16);
  a.ent = reinterpret_cast<const uint2*>(base + L.ent);
  a.partial = reinterpret_cast<float*>(base + L.partial);
  a.B = B; a.ldb = ldb; a.kmax = kmax;
  a.ent_cap = (int32_t)std::max<int64_t>(p.entries, 1);
  const size_t lds = 2 * (size_t)kTileBuf + (size_t)kTileWaves * 128 * sizeof(uint2);   // tiles + entry rings
  auto go = [&](auto kern, auto comb) -> int {
    SAGNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)lds));
    hipLaunchKernelGGL(kern, dim3((unsigned)p.n_items), dim3(kTileWaves * 64), lds, s, a);
    SAGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(comb, dim3((unsigned)ceil_div(p.rows, kT / 64)), dim3(kT), 0, s, a.hdr, generation,
                       P32(L.hubrow), P32(L.group_item0), a.partial, (int32_t)p.rows, (int32_t)g.rg, m, C, ldc);
    SAGNN_LAUNCH_CHECK();
    return SAGNN_OK;
  };
  if (f == 64) return go(tile_spmm_kernel<1, 32>, tile_combine_kernel<1>);
  if (f == 128) return go(tile_spmm_kernel<2, 32>, tile_combine_kernel<2>);
  return go(tile_spmm_kernel<4, 16>, tile_combine_kernel<4>);
}

}  // namespace sagnn
