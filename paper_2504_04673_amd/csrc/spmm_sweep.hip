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
// Pieces of a split row are summed in a fixed order by a small second kernel.  Short rows go
// through the nonzero-splitting kernels of spmm.hip on a compacted CSR.
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
#include <queue>
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

// One workgroup per wavefront: segment the 16 pieces by slab, lay the entries out in
// (slab, piece) order and encode them.  With `groups` = R lane groups the wavefront carries R
// independent streams (group g owns slots g*16/R ..), stored zipped: entry t of group g at
// position R*t + g; the shorter streams are padded with entries that multiply row 0 of B by 0.
__global__ __launch_bounds__(kBuildThreads) void sweep_build_kernel(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
    const float* __restrict__ val, const int32_t* __restrict__ piece_info,
    const int32_t* __restrict__ wave_base, int32_t n_slabs, int32_t slab_width, uint32_t kmax,
    int32_t stagger, int32_t groups, uint32_t* __restrict__ code, float* __restrict__ vals) {
  // dynamic LDS (sweep_build_lds_bytes): lo[16][S+1] first entry (index in row) of slab s;
  // off[S][16] offset of segment (s, slot) inside its slab; slab_base[S][16] stream offset of
  // slab s for group g; slab_tot[S][16]
  extern __shared__ __attribute__((aligned(16))) int32_t build_lds[];
  const int SS = n_slabs;
  int32_t* lo_ = build_lds;                                  // [16][SS + 1]
  int32_t* off_ = lo_ + kSweepSlots * (SS + 1);              // [SS][16]
  int32_t* slab_base_ = off_ + SS * kSweepSlots;             // [SS][16]
  int32_t* slab_tot_ = slab_base_ + SS * kSweepSlots;        // [SS][16]
#define LO(slot, s) lo_[(slot) * (SS + 1) + (s)]
#define OFF(s, slot) off_[(s) * kSweepSlots + (slot)]
#define SLAB_BASE(s, g) slab_base_[(s) * kSweepSlots + (g)]
#define SLAB_TOT(s, g) slab_tot_[(s) * kSweepSlots + (g)]
  __shared__ int32_t glen[kSweepSlots];
  __shared__ int32_t p_row[kSweepSlots], p_j[kSweepSlots], p_p[kSweepSlots], p_beg[kSweepSlots],
      p_deg[kSweepSlots];
  const int64_t w = blockIdx.x;
  const int tid = threadIdx.x;
  const int S = n_slabs;
  const int R = groups, SL = kSweepSlots / groups;
  if (tid < kSweepSlots) {
    const int32_t row = piece_info[2 * (w * kSweepSlots + tid)];
    const int32_t jp = piece_info[2 * (w * kSweepSlots + tid) + 1];
    p_row[tid] = row;
    p_j[tid] = jp >> 16;
    p_p[tid] = jp & 0xFFFF;
    p_beg[tid] = row >= 0 ? rowptr[row] : 0;
    p_deg[tid] = row >= 0 ? rowptr[row + 1] - rowptr[row] : 0;
  }
  __syncthreads();
  for (int idx = tid; idx < kSweepSlots * (S + 1); idx += kBuildThreads) {
    const int slot = idx / (S + 1), s = idx - slot * (S + 1);
    int32_t res = 0;
    if (p_row[slot] >= 0) {
      const int32_t d = p_deg[slot];
      if (s == S) {
        res = d;
      } else {
        // lower bound of column s*slab_width in the (ascending) row
        const int64_t target = (int64_t)s * slab_width;
        const int32_t* __restrict__ c = colidx + p_beg[slot];
        int32_t a = 0, b = d;
        while (a < b) {
          const int32_t mid = (a + b) >> 1;
          const uint32_t cv = (uint32_t)c[mid] > kmax ? kmax : (uint32_t)c[mid];
          if ((int64_t)cv < target) a = mid + 1; else b = mid;
        }
        res = a;
      }
    }
    LO(slot, s) = res;
  }
  __syncthreads();
  // entries of segment (s, slot); then per slab the prefix over the slots of each group
  for (int idx = tid; idx < S * kSweepSlots; idx += kBuildThreads) {
    const int s = idx / kSweepSlots, slot = idx - s * kSweepSlots;
    OFF(s, slot) = p_row[slot] >= 0 ? count_upto(LO(slot, s + 1), p_j[slot], p_p[slot]) -
                                          count_upto(LO(slot, s), p_j[slot], p_p[slot])
                                    : 0;
  }
  __syncthreads();
  for (int idx = tid; idx < S * R; idx += kBuildThreads) {
    const int s = idx / R, gi = idx - s * R;
    int32_t run = 0;
    for (int slot = gi * SL; slot < (gi + 1) * SL; ++slot) {
      const int32_t c = OFF(s, slot);
      OFF(s, slot) = run;
      run += c;
    }
    SLAB_TOT(s, gi) = run;
  }
  __syncthreads();
  // The stream is laid out in the order the wavefront will walk the slabs: it starts at slab
  // s0 = xcd * S/8 (xcd = workgroup index mod 8, four wavefronts per workgroup) and wraps.
  const int s0 = stagger ? (int)(((w >> 2) & 7) * S / 8) : 0;
  if (tid < R) {
    int32_t run = 0;
    for (int t = 0; t < S; ++t) {
      const int s = (s0 + t) % S;
      SLAB_BASE(s, tid) = run;
      run += SLAB_TOT(s, tid);
    }
    glen[tid] = run;
  }
  __syncthreads();
  const int64_t base = wave_base[w];
  const int64_t steps = (wave_base[w + 1] - base) / R;     // padded length of every group stream
  for (int gi = 0; gi < R; ++gi)
    for (int64_t t = glen[gi] + tid; t < steps; t += kBuildThreads) {
      code[base + t * R + gi] = 0u;
      vals[base + t * R + gi] = 0.f;
    }
  for (int slot = 0; slot < kSweepSlots; ++slot) {
    if (p_row[slot] < 0) continue;
    const int gi = slot / SL;
    const int32_t j = p_j[slot], p = p_p[slot], d = p_deg[slot], beg = p_beg[slot];
    const int32_t size = count_upto(d, j, p);
    for (int32_t t = tid; t < size; t += kBuildThreads) {
      const int32_t i = j + t * p;
      const uint32_t craw = (uint32_t)colidx[beg + i];
      const uint32_t c = craw > kmax ? kmax : craw;
      int s = (int)(c / (uint32_t)slab_width);
      if (s > S - 1) s = S - 1;
      // the row is ascending, but clamped / equal columns may sit on a slab boundary: trust lo[]
      while (s > 0 && i < LO(slot, s)) --s;
      while (s < S - 1 && i >= LO(slot, s + 1)) ++s;
      const int32_t rank = t - count_upto(LO(slot, s), j, p);
      // a segment also ends every kSweepRunMax entries, which bounds the length of any serial
      // fp32 accumulation (and with it the rounding bias on rows of equal terms)
      const bool last = i + p >= LO(slot, s + 1) || (rank & (kSweepRunMax - 1)) == kSweepRunMax - 1;
      const int64_t pos = base + (int64_t)(SLAB_BASE(s, gi) + OFF(s, slot) + rank) * R + gi;
      code[pos] = c | ((uint32_t)slot << kSweepColBits) | (last ? 0x80000000u : 0u);
      vals[pos] = val[beg + i];
    }
  }
}
#undef LO
#undef OFF
#undef SLAB_BASE
#undef SLAB_TOT

inline size_t sweep_build_lds_bytes(int64_t S) {
  return sizeof(int32_t) * (size_t)(kSweepSlots * (S + 1) + 3 * S * kSweepSlots);
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
};

template <int FPL, int U, bool BUF>
__global__ __launch_bounds__(256) void spmm_sweep_kernel(
    const uint32_t* __restrict__ code, const float* __restrict__ vals,
    const int32_t* __restrict__ wave_base, const int32_t* __restrict__ piece_target,
    const SpmmWsHeader* __restrict__ hdr, const float* __restrict__ B, float* __restrict__ C,
    float* __restrict__ partial, const SweepDims d) {
  using vec = typename Vec<FPL>::T;
  extern __shared__ __attribute__((aligned(16))) float lds_acc[];  // [4 waves][16 slots][64*FPL]
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t loff = lane * (FPL * 4);
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int64_t w = (int64_t)blockIdx.x * 4 + wave;
  if (w >= d.n_waves) return;
  if (hdr->magic != kSpmmMagic || hdr->generation != d.generation || hdr->n_waves != d.n_waves ||
      hdr->groups != 1)
    return;
  constexpr int kRow = 64 * FPL;  // floats per accumulator row
  float* __restrict__ my = lds_acc + (size_t)wave * kSweepSlots * kRow + lane * FPL;
#pragma unroll
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
      if (c[u] >> 31) {   // last entry of a (piece, slab) segment: fold into the piece's LDS row
        vec* p = reinterpret_cast<vec*>(my + ((c[u] >> kSweepColBits) & (kSweepSlots - 1)) * kRow);
        *p += acc;
        acc = 0.f;
      }
    }
  }

#pragma unroll 1
  for (int s = 0; s < kSweepSlots; ++s) {
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

// Lane-group variant: the wavefront carries R independent streams (zipped in memory), lane
// group g = lanes [g*64/R, (g+1)*64/R) walks stream g.  A group's 64/R lanes move one whole row
// of B with V floats (16 bytes at V = 4) per lane, so one load instruction serves R entries.
// Column ids and values still arrive by scalar loads; a lane picks its group's pair with
// selects (the row offset is multiplied on the scalar side first).  Flushes are per group:
// lanes of other groups are masked off by the divergent branch.
template <int V, int R, int U, bool BUF>
__global__ __launch_bounds__(256) void spmm_sweep_group_kernel(
    const uint32_t* __restrict__ code, const float* __restrict__ vals,
    const int32_t* __restrict__ wave_base, const int32_t* __restrict__ piece_target,
    const SpmmWsHeader* __restrict__ hdr, const float* __restrict__ B, float* __restrict__ C,
    float* __restrict__ partial, const SweepDims d) {
  using vec = typename Vec<V>::T;
  constexpr int LG = 64 / R;             // lanes per group = lanes per row
  constexpr int kRow = LG * V;           // floats per row of this launch
  constexpr int SL = kSweepSlots / R;    // slots per group
  extern __shared__ __attribute__((aligned(16))) float lds_acc[];  // [4 waves][16 slots][kRow]
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t gid = lane / LG, lig = lane % LG;
  const uint32_t loff = lig * (V * 4);
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int64_t w = (int64_t)blockIdx.x * 4 + wave;
  if (w >= d.n_waves) return;
  if (hdr->magic != kSpmmMagic || hdr->generation != d.generation || hdr->n_waves != d.n_waves ||
      hdr->groups != R)
    return;
  float* __restrict__ my = lds_acc + (size_t)wave * kSweepSlots * kRow + lig * V;
#pragma unroll
  for (int ls = 0; ls < SL; ++ls) *reinterpret_cast<vec*>(my + (gid * SL + ls) * kRow) = vec(0.f);

  const int32_t base = wave_base[w];
  const int32_t steps = (wave_base[w + 1] - base) / R;   // a multiple of U (padded when built)
  const uint32_t* __restrict__ cw = code + base;
  const float* __restrict__ vw = vals + base;
  const __amdgpu_buffer_rsrc_t rs = make_rsrc(B, d.b_bytes);

  vec acc = 0.f;
  for (int32_t e = 0; e < steps; e += U) {
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

#pragma unroll 1
  for (int ls = 0; ls < SL; ++ls) {
    const int slot = (int)gid * SL + ls;
    const int32_t tgt = piece_target[w * kSweepSlots + slot];
    if (tgt == INT32_MIN) continue;
    vec r = *reinterpret_cast<const vec*>(my + slot * kRow);
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

int env_int(const char* name, int dflt) {
  const char* v = getenv(name);
  return v ? atoi(v) : dflt;
}

struct Piece {
  int32_t size, row, j, p;
};

std::atomic<uint64_t> g_generation{1};
thread_local SweepTuning g_tuning{0, 0};

}  // namespace

void sweep_set_tuning(SweepTuning t) { g_tuning = t; }

// ---------------------------------------------------------------------------------------
// host side of the preparation: classify rows, cut long rows into pieces, deal pieces to the
// streams of the wavefronts (largest first, each to the shortest stream so far, so the streams
// have nearly equal lengths), build the compacted short-row CSR.
int sweep_prepare(const int32_t* d_rowptr, const int32_t* d_colidx, const float* d_val, int64_t m,
                  int64_t k, int64_t nnz, int32_t f, char* ws, const SpmmWsLayout& L,
                  hipStream_t s, SweepPlanResult* out) {
  out->use_sweep = false;
  const int force = env_int("SAGNN_SWEEP", -1);  // 0: never, 1: whenever possible, -1: heuristic
  if (force == 0 || nnz < 4096 || k <= 0 || k >= (1ll << kSweepColBits) || m <= 0) return SAGNN_OK;
  const int64_t b_bytes = k * (int64_t)f * 4;
  // worth it only if B is much larger than an L2 (the long-row share is checked below)
  if (force != 1 && (nnz < (1 << 20) || b_bytes <= (8ll << 20))) return SAGNN_OK;

  std::vector<int32_t> rp((size_t)m + 1);
  SAGNN_HIP(hipMemcpyAsync(rp.data(), d_rowptr, sizeof(int32_t) * (size_t)(m + 1),
                           hipMemcpyDeviceToHost, s));
  SAGNN_HIP(hipStreamSynchronize(s));
  if (rp[0] != 0 || rp[m] != nnz) return SAGNN_OK;  // inconsistent: keep the plain schedule

  // Rows with at least min_long entries go through the sweep.  64 suits power-law graphs (the
  // many rows below it hold few entries and would only add accumulator slots); when the rows of
  // 16..63 entries hold a large share of the matrix (near-regular graphs, e.g. a partitioned
  // graph's row block) the threshold drops so that they are swept too.
  int min_long = env_int("SAGNN_SWEEP_MINDEG", 0);
  if (min_long <= 0) {
    int64_t mid = 0;
    for (int64_t r = 0; r < m; ++r) {
      const int64_t d = (int64_t)rp[r + 1] - rp[r];
      if (d >= kSweepMinLong && d < 64) mid += d;
    }
    min_long = (mid * 4 >= nnz) ? kSweepMinLong : (g_tuning.min_long > 0 ? g_tuning.min_long : 64);
  }
  if (min_long < kSweepMinLong) min_long = kSweepMinLong;
  int piece_max = env_int("SAGNN_SWEEP_PIECE", g_tuning.piece > 0 ? g_tuning.piece : 4096);
  if (piece_max < 1024) piece_max = 1024;
  if (piece_max > 32768) piece_max = 32768;
  const int64_t slab_bytes = (int64_t)env_int("SAGNN_SWEEP_SLAB_MB", 4) << 20;
  int64_t S = slab_bytes >= (1 << 16) ? 8 * ceil_div(b_bytes, 8 * slab_bytes) : kSweepMaxSlabs;
  if (S < 8) S = 8;
  if (S > kSweepMaxSlabs) S = kSweepMaxSlabs;
  const int64_t width = ceil_div(k, S);

  // Lane groups: at f = 128 half a wavefront, at f = 64 a quarter, moves a whole row of B with
  // 16 bytes per lane, so one load instruction serves 2 / 4 entries (the vector-memory issue
  // rate, not bandwidth, bounds B-in-cache cases).  Other widths keep one row per instruction.
  // They pay when the rows of B are re-used from cache (issue-bound: 233 k-vertex graph
  // 3.38 -> 2.63 ms, 2.45 M-vertex graph 4.85 -> 4.62 ms) and cost ~3 % when almost every gather
  // misses (rank share of the 111 M-vertex graph, 2.6 entries per row of B): decided below by
  // the average number of swept entries per row of B.
  // Narrow operands (f = 32, 16: rows of 128 / 64 bytes, 8 / 4 lanes each) exist only in the
  // grouped form, 8 / 16 rows per load.
  int64_t R = f == 128 ? 2 : (f == 64 ? 4 : (f == 32 ? 8 : (f == 16 ? 16 : 1)));
  const int groups_env = env_int("SAGNN_SWEEP_GROUPS", 0);   // 1: never, 2: whenever possible
  if (groups_env == 1 && f >= 64) R = 1;
  std::vector<Piece> pieces;
  int64_t long_entries = 0, short_rows = 0, short_entries = 0;
  bool has_empty = false;
  for (int64_t r = 0; r < m; ++r) {
    const int64_t d = (int64_t)rp[r + 1] - rp[r];
    if (d < 0) return SAGNN_OK;
    if (d == 0) { has_empty = true; continue; }
    if (d >= min_long) {
      const int32_t p = (int32_t)ceil_div(d, piece_max);
      if (p > 0x7FFF) return SAGNN_OK;
      for (int32_t j = 0; j < p; ++j)
        pieces.push_back({(int32_t)((d - j + p - 1) / p), (int32_t)r, j, p});
      long_entries += d;
    } else {
      ++short_rows;
      short_entries += d;
    }
  }
  if (force != 1 && long_entries * 10 < nnz * 3) return SAGNN_OK;   // < 30 % of the entries
  if (groups_env != 2 && long_entries < 8 * k) {
    if (f < 64) return SAGNN_OK;   // no one-row-per-instruction form below 64: plain schedule
    R = 1;
  }
  if (pieces.empty() || (int64_t)pieces.size() > L.max_pieces) return SAGNN_OK;

  std::vector<char> is_long((size_t)m, 0);
  for (const Piece& pc : pieces) is_long[(size_t)pc.row] = 1;
  const int64_t P = (int64_t)pieces.size();
  // Pieces per wavefront: all kSweepSlots when there are plenty of pieces; fewer when that would
  // leave the chip short of wavefronts (a row block of a partitioned graph has few long rows).
  int64_t slots_used = ceil_div(P, (int64_t)env_int("SAGNN_SWEEP_MIN_WAVES", 8192));
  if (slots_used < R) slots_used = R;          // every lane group of a wavefront gets a piece
  if (slots_used > kSweepSlots) slots_used = kSweepSlots;
  if (ceil_div(P, slots_used) + 64 > L.max_waves - 1) slots_used = kSweepSlots;
  // Pieces are dealt window by window.  A window is a run of consecutive long rows holding a
  // few times as many pieces as the chip keeps resident at once (LDS-limited); inside a window
  // the pieces are sorted by size and dealt longest-first, so its wavefronts have nearly equal
  // stream lengths (they pass the slabs in step).  A matrix of up to ~4 generations is one
  // window (measured best on randomly labelled graphs: 4.95 ms against 5.4 ms with one window
  // per generation on the 2.45 M-vertex R-MAT graph); a larger one whose row order carries
  // locality (a partitioned graph) keeps it, because a window only touches the part of B its
  // rows' neighbourhoods live in (2 M-vertex community-ordered graph: 13.9 -> 11.4 ms).
  const int64_t lds_per_wg = 4ll * kSweepSlots * f * 4;
  int64_t wg_per_cu = (160 * 1024) / lds_per_wg;
  if (wg_per_cu > 8) wg_per_cu = 8;
  if (wg_per_cu < 1) wg_per_cu = 1;
  const int64_t resident_waves = 256 * wg_per_cu * 4;
  int64_t window = resident_waves * slots_used;              // pieces per window
  {
    const int pct = env_int("SAGNN_SWEEP_WINDOW_PCT", 400);  // 0: one window (global dealing)
    window = pct <= 0 ? P : std::max<int64_t>(slots_used, window * pct / 100);
  }
  std::vector<int64_t> win_wave0;                            // first wavefront of every window
  int64_t NW = 0;
  for (int64_t a = 0; a < P; a += window) {
    const int64_t b = std::min(P, a + window);
    std::sort(pieces.begin() + a, pieces.begin() + b, [](const Piece& x, const Piece& y) {
      if (x.size != y.size) return x.size > y.size;
      if (x.row != y.row) return x.row < y.row;
      return x.j < y.j;
    });
    win_wave0.push_back(NW);
    // wavefronts of this window: as many as keep the stream length equal to the global average
    // (equal lengths in ALL windows keep successive generations in step), but never fewer than
    // the slots allow
    int64_t entries_w = 0;
    for (int64_t t = a; t < b; ++t) entries_w += pieces[(size_t)t].size;
    const double target_len = (double)long_entries / (double)ceil_div(P, slots_used);
    int64_t nw = (int64_t)((double)entries_w / target_len + 0.5);
    nw = std::max(nw, ceil_div(b - a, (int64_t)kSweepSlots));
    nw = std::max<int64_t>(nw, 1);
    nw = std::min(nw, b - a);
    NW += nw;
  }
  win_wave0.push_back(NW);
  if (NW > L.max_waves - 1) return SAGNN_OK;   // cannot happen with the bounds above; plain schedule
  std::vector<int32_t> info((size_t)NW * kSweepSlots * 2, -1), target((size_t)NW * kSweepSlots, INT32_MIN);
  // multi-piece rows: partial slots in row order
  std::vector<int32_t> multi_row, multi_first;
  {
    std::vector<std::pair<int32_t, int32_t>> mr;  // (row, p)
    for (const Piece& pc : pieces)
      if (pc.p > 1 && pc.j == 0) mr.push_back({pc.row, pc.p});
    std::sort(mr.begin(), mr.end());
    multi_first.push_back(0);
    for (auto& e : mr) {
      multi_row.push_back(e.first);
      multi_first.push_back(multi_first.back() + e.second);
    }
  }
  if ((int64_t)multi_row.size() > L.max_multi_rows || (int64_t)multi_first.back() > L.max_multi_pieces)
    return SAGNN_OK;
  // Inside a window: largest piece first, each to the stream that is shortest so far and still
  // has a free slot (ties: lowest index).  Streams come out equal to within a piece of the
  // smallest size class, which keeps the wavefronts in step from slab to slab.  With R lane
  // groups a wavefront carries R independent streams (group g owns slots g*16/R ..); the unit of
  // dealing is then the group stream.
  const int64_t SL = kSweepSlots / R;           // slots per group stream
  std::vector<int32_t> used((size_t)NW * R, 0);
  std::vector<int64_t> uload((size_t)NW * R, 0);
  using Load = std::pair<int64_t, int64_t>;   // (stream length, unit = wavefront * R + group)
  std::priority_queue<Load, std::vector<Load>, std::greater<Load>> heap;
  int64_t cur_win = -1;
  const bool lpt = R > 1 || env_int("SAGNN_SWEEP_LPT", 1) != 0;
  for (int64_t t = 0; t < P; ++t) {
    const int64_t win = t / window, tw = t - win * window;
    const int64_t nw = win_wave0[(size_t)win + 1] - win_wave0[(size_t)win];
    int64_t wv, slot;
    if (lpt) {
      if (win != cur_win) {
        cur_win = win;
        heap = decltype(heap)();
        for (int64_t u = 0; u < nw * R; ++u) heap.push({0, win_wave0[(size_t)win] * R + u});
      }
      if (heap.empty()) return SAGNN_EINVAL;   // nw * kSweepSlots >= pieces of the window
      const int64_t unit = heap.top().second;
      heap.pop();
      wv = unit / R;
      slot = (unit % R) * SL + used[(size_t)unit]++;
      uload[(size_t)unit] += pieces[(size_t)t].size;
      if (used[(size_t)unit] < SL) heap.push({uload[(size_t)unit], unit});
    } else {
      slot = tw / nw;
      const int64_t pos = tw % nw;
      wv = win_wave0[(size_t)win] + ((slot & 1) ? nw - 1 - pos : pos);
      uload[(size_t)wv] += pieces[(size_t)t].size;
    }
    const size_t g = (size_t)(wv * kSweepSlots + slot);
    const Piece& pc = pieces[(size_t)t];
    info[2 * g] = pc.row;
    info[2 * g + 1] = (pc.j << 16) | pc.p;
    if (pc.p == 1) {
      target[g] = pc.row;
    } else {
      const size_t q = (size_t)(std::lower_bound(multi_row.begin(), multi_row.end(), pc.row) - multi_row.begin());
      target[g] = -(multi_first[q] + pc.j) - 1;
    }
  }
  // A wavefront's R group streams are stored zipped (entry t of group g at R*t + g), each padded
  // to the longest of them and to a multiple of the kernel's batch (8 steps)
  std::vector<int32_t> wbase((size_t)NW + 1);
  int64_t run = 0, unpadded = 0;
  for (int64_t wv = 0; wv < NW; ++wv) {
    wbase[(size_t)wv] = (int32_t)run;
    int64_t longest = 0;
    for (int64_t gi = 0; gi < R; ++gi) {
      longest = std::max(longest, uload[(size_t)(wv * R + gi)]);
      unpadded += uload[(size_t)(wv * R + gi)];
    }
    run += (longest + 7) / 8 * 8 * R;
    if (run > 0x7FFFFFF0ll) return SAGNN_OK;
  }
  wbase[(size_t)NW] = (int32_t)run;
  if (unpadded != long_entries) return SAGNN_EINVAL;
  const int64_t stream_len = run;
  const int64_t short_base = round_up((size_t)stream_len + 64, 256);
  if (short_base + short_entries + kSpmmChunk > L.stream_cap) return SAGNN_OK;

  // short-row CSR
  std::vector<int32_t> rps((size_t)short_rows + 1), rmap((size_t)short_rows + 1);
  {
    int64_t i = 0, acc = 0;
    for (int64_t r = 0; r < m; ++r) {
      const int64_t d = (int64_t)rp[r + 1] - rp[r];
      if (d > 0 && !is_long[(size_t)r]) { rps[(size_t)i] = (int32_t)acc; rmap[(size_t)i] = (int32_t)r; acc += d; ++i; }
    }
    rps[(size_t)short_rows] = (int32_t)acc;
  }

  auto up = [&](size_t off, const void* src, size_t bytes) {
    return bytes ? hipMemcpyAsync(ws + off, src, bytes, hipMemcpyHostToDevice, s) : hipSuccess;
  };
  SAGNN_HIP(up(L.piece_info, info.data(), info.size() * 4));
  SAGNN_HIP(up(L.piece_target, target.data(), target.size() * 4));
  SAGNN_HIP(up(L.wave_base, wbase.data(), wbase.size() * 4));
  SAGNN_HIP(up(L.multi_row, multi_row.data(), multi_row.size() * 4));
  SAGNN_HIP(up(L.multi_first, multi_first.data(), multi_first.size() * 4));
  SAGNN_HIP(up(L.rowptr_s, rps.data(), rps.size() * 4));
  SAGNN_HIP(up(L.rowmap_s, rmap.data(), rmap.size() * 4));

  // long rows must be column-sorted for the slab segmentation
  int32_t* d_flag = reinterpret_cast<int32_t*>(ws + L.carry);  // scratch until the first product
  SAGNN_HIP(hipMemsetAsync(d_flag, 0, 4, s));
  hipLaunchKernelGGL(sweep_check_sorted_kernel, dim3((unsigned)ceil_div(NW * kSweepSlots, 4)), dim3(256),
                     0, s, d_rowptr, d_colidx, reinterpret_cast<const int32_t*>(ws + L.piece_info),
                     NW * kSweepSlots, (uint32_t)(k - 1), d_flag);
  SAGNN_LAUNCH_CHECK();
  int32_t unsorted = 0;
  SAGNN_HIP(hipMemcpyAsync(&unsorted, d_flag, 4, hipMemcpyDeviceToHost, s));
  SAGNN_HIP(hipStreamSynchronize(s));
  if (unsorted) return SAGNN_OK;

  const uint32_t kmax = (uint32_t)(k - 1);
  const size_t build_lds = sweep_build_lds_bytes(S);
  SAGNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(sweep_build_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)build_lds));
  hipLaunchKernelGGL(sweep_build_kernel, dim3((unsigned)NW), dim3(kBuildThreads), build_lds, s, d_rowptr, d_colidx,
                     d_val, reinterpret_cast<const int32_t*>(ws + L.piece_info),
                     reinterpret_cast<const int32_t*>(ws + L.wave_base), (int32_t)S, (int32_t)width, kmax,
                     (int32_t)env_int("SAGNN_SWEEP_STAGGER", 0), (int32_t)R,
                     reinterpret_cast<uint32_t*>(ws + L.code), reinterpret_cast<float*>(ws + L.vals));
  SAGNN_LAUNCH_CHECK();
  // zero the gap between the long stream and the short entries (tail batches read into it)
  SAGNN_HIP(hipMemsetAsync(ws + L.code + 4 * (size_t)stream_len, 0, 4 * (size_t)(short_base - stream_len), s));
  SAGNN_HIP(hipMemsetAsync(ws + L.vals + 4 * (size_t)stream_len, 0, 4 * (size_t)(short_base - stream_len), s));
  if (short_rows > 0) {
    hipLaunchKernelGGL(sweep_short_copy_kernel, dim3((unsigned)ceil_div(short_rows, 256)), dim3(256), 0, s,
                       d_rowptr, d_colidx, d_val, reinterpret_cast<const int32_t*>(ws + L.rowptr_s),
                       reinterpret_cast<const int32_t*>(ws + L.rowmap_s), short_rows,
                       reinterpret_cast<int32_t*>(ws + L.code) + short_base,
                       reinterpret_cast<float*>(ws + L.vals) + short_base);
    SAGNN_LAUNCH_CHECK();
  }
  SAGNN_HIP(hipStreamSynchronize(s));  // host vectors are read by the copies above

  SpmmWsHeader& h = out->hdr;
  h = SpmmWsHeader{};
  h.magic = kSpmmMagic;
  h.has_empty_rows = has_empty ? 1 : 0;
  h.m = m; h.nnz = nnz; h.f = f; h.mode = 1;
  h.generation = g_generation.fetch_add(1);
  h.c_rows = short_rows; h.c_nnz = short_entries; h.c_nchunks = spmm_nchunks(short_entries);
  h.n_waves = NW; h.n_long_entries = stream_len;   // padded length of the sweep streams
  h.n_multi_rows = (int64_t)multi_row.size(); h.n_multi_pieces = multi_first.back();
  h.n_slabs = (int32_t)S; h.slab_width = (int32_t)width;
  h.groups = (int32_t)R;
  out->use_sweep = true;
  return SAGNN_OK;
}

uint64_t spmm_next_generation() { return g_generation.fetch_add(1); }

int sweep_launch(const SpmmHostDesc& d, const SpmmWsLayout& L, char* ws, const float* B,
                 int64_t ldb, int32_t col0, int32_t fw, uint32_t kmax, float* C, int64_t ldc,
                 int32_t accumulate, int32_t f_total, hipStream_t s) {
  if (d.n_waves <= 0) return SAGNN_OK;
  SweepDims sd{};
  sd.n_waves = d.n_waves; sd.ldb = ldb; sd.ldc = ldc; sd.f_total = f_total;
  sd.generation = d.generation; sd.col0 = col0; sd.accumulate = accumulate;
  // bytes of B reachable from B + col0: rows 0..kmax, fw columns each (columns were clamped to
  // kmax when the stream was built)
  sd.b_bytes = 0;
  const bool buf = buffer_addressable(kmax, ldb, fw, &sd.b_bytes);
  sd.row_bytes = (uint32_t)(ldb * 4);
  const unsigned blocks = (unsigned)ceil_div(d.n_waves, 4);
  const size_t lds = (size_t)4 * kSweepSlots * fw * sizeof(float);
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
  if (d.groups == 16)    // prepared for f = 16: four lanes per row
    return fw == 16 ? (buf ? go(spmm_sweep_perm_kernel<16, true>) : go(spmm_sweep_perm_kernel<16, false>))
                    : SAGNN_EINVAL;
  if (d.groups == 8)     // prepared for f = 32: eight lanes per row
    return fw == 32 ? (buf ? go(spmm_sweep_perm_kernel<8, true>) : go(spmm_sweep_perm_kernel<8, false>))
                    : SAGNN_EINVAL;
  if (d.groups == 2) {   // prepared for f = 128: half a wavefront per row (or per half row at 64)
    if (fw == 128) return buf ? go(spmm_sweep_group_kernel<4, 2, 8, true>) : go(spmm_sweep_group_kernel<4, 2, 8, false>);
    if (fw == 64) return buf ? go(spmm_sweep_group_kernel<2, 2, 8, true>) : go(spmm_sweep_group_kernel<2, 2, 8, false>);
    return SAGNN_EINVAL;
  }
  if (d.groups == 4) {   // prepared for f = 64: a quarter wavefront per row
    if (fw == 64) return buf ? go(spmm_sweep_group_kernel<4, 4, 8, true>) : go(spmm_sweep_group_kernel<4, 4, 8, false>);
    return SAGNN_EINVAL;
  }
  if (fw == 256) return buf ? go(spmm_sweep_kernel<4, 8, true>) : go(spmm_sweep_kernel<4, 8, false>);
  if (fw == 128) return buf ? go(spmm_sweep_kernel<2, 8, true>) : go(spmm_sweep_kernel<2, 8, false>);
  if (fw == 64) return buf ? go(spmm_sweep_kernel<1, 8, true>) : go(spmm_sweep_kernel<1, 8, false>);
  return SAGNN_EINVAL;
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
