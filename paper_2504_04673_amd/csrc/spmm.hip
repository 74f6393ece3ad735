// Local CSR x tall-skinny dense product  C (+)= A * B  (Alg. 1 / Alg. 2, the statement
// "Z <- Z + SpMM(A_iq, H^)"; Sec. 4.1 block-sum equation).  fp32 FMA on the vector ALUs.
//
// Schedule: nonzero splitting.  The nnz stored entries are cut into chunks of kSpmmChunk
// consecutive entries; one wavefront owns one chunk, whatever rows it covers, so a hub row of
// a power-law graph is spread over many wavefronts and a run of short rows shares one.
// Because the sparsity pattern is fixed for the whole training run, spmm_csr_prepare() records
// once (a) the row in which each chunk starts and (b) one bit per entry telling whether the
// entry is the last of its row.  The product kernel then walks its chunk as a flat stream:
// the column indices and values of a batch are wavefront-uniform (scalar loads), the 64
// lanes split the f columns of the dense row (coalesced 64*FPL*4-byte reads along f), all
// loads of a batch are issued before the first FMA, and a set "row end" bit flushes the
// accumulator to C.  A row that started in an earlier chunk is flushed to a per-chunk carry
// slot instead; a second small kernel adds the carries to C in chunk order, so the result is
// reproducible (no floating-point atomics).
//
// Narrow matrices (f < 64) use sub-wavefront groups: G = f/4 lanes (rounded up to a power of
// two) read one dense row as float4 pieces, and 64/G entries are processed per step; a row
// end inside a step triggers a cross-group butterfly reduction.
//
// Widths other than 64/128/256 are processed as column slabs of those widths plus a narrow
// remainder.
#include <stdlib.h>


#include "common.h"
#include "rowload.h"

namespace sagnn {
namespace {

constexpr int kT = kSpmmChunk;
constexpr int kWavesPerBlock = 4;
constexpr int kBlock = kWavesPerBlock * 64;

// Scalars of a launch.  Pointers are passed as separate __restrict__ kernel parameters: that
// is what lets the compiler prove the index/value streams are never written by the kernel and
// fetch them with scalar loads.
struct SpmmDims {
  int64_t m, nnz, nchunks, ldb, ldc, carry_ld;  // m, nnz, nchunks: of the CSR being walked
  uint64_t generation;
  uint32_t b_bytes;    // bytes addressable from B (buffer-load variant)
  uint32_t row_bytes;  // ldb * 4
  uint32_t kmax;  // k - 1: largest valid column index
  int32_t f;      // columns handled by this launch (slab width)
  int32_t accumulate;
};

__device__ __forceinline__ bool ws_matches(const SpmmWsHeader* __restrict__ hdr, const SpmmDims& d) {
  return hdr->magic == kSpmmMagic && hdr->generation == d.generation && hdr->c_rows == d.m &&
         hdr->c_nnz == d.nnz && hdr->c_nchunks == d.nchunks;
}

__device__ __forceinline__ int next_row(int r, bool has_empty, const int32_t* __restrict__ rowptr,
                                        int64_t m) {
  ++r;
  if (has_empty)
    while (r < m - 1 && rowptr[r + 1] == rowptr[r]) ++r;
  return r;
}

#define SPMM_PTR_PARAMS                                                                     \
  const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,                   \
      const float *__restrict__ val, const float *__restrict__ B, float *__restrict__ C,    \
      const SpmmWsHeader *__restrict__ hdr, const int32_t *__restrict__ chunk_row,          \
      const uint32_t *__restrict__ flags, float *__restrict__ carry_base,                   \
      const int32_t *__restrict__ rowmap

// ------------------------------------------------------------------------------------------
// wide kernel: f == 64 * FPL, one entry per wavefront load.
// Per batch of U entries: U dense-row loads are issued back to back (their column indices and
// values are already in scalar registers), then the scalar loads of the NEXT batch, then the
// FMAs with a uniform branch at every row end.
template <int FPL, int U, bool BUF, bool AHEAD>
__global__ __launch_bounds__(kBlock) void spmm_wide_kernel(SPMM_PTR_PARAMS, const SpmmDims d) {
  using vec = typename Vec<FPL>::T;
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t loff = lane * (FPL * 4);  // byte offset of this lane's columns inside a row
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int64_t k = (int64_t)blockIdx.x * kWavesPerBlock + wave;
  if (k >= d.nchunks) return;
  if (!ws_matches(hdr, d)) return;
  const bool has_empty = hdr->has_empty_rows != 0 && rowmap == nullptr;
  const int32_t e0 = (int32_t)(k * kT);
  const int32_t e1 = (int32_t)((d.nnz - e0 < kT) ? d.nnz : e0 + kT);
  int r = chunk_row[k];
  r = r < 0 ? 0 : (r > d.m - 1 ? (int)(d.m - 1) : r);
  bool head = rowptr[r] < e0;  // first row began in an earlier chunk -> carry slot
  const uint32_t* __restrict__ fl = flags + (e0 >> 5);
  char* __restrict__ carry = reinterpret_cast<char*>(carry_base + k * d.carry_ld) + loff;
  const __amdgpu_buffer_rsrc_t rs = make_rsrc(B, d.b_bytes);

  vec acc = 0.f;
  // `old` = the current contents of the row of C when they were fetched ahead (accumulating
  // calls), otherwise they are read here
  auto flush = [&](const vec old, const bool have_old) {
    if (r >= d.m) return;  // cannot happen with a consistent rowptr; keeps stores in bounds
    if (head) {
      *reinterpret_cast<vec*>(carry) = acc;
      head = false;
    } else {
      const int64_t ro = rowmap ? rowmap[r] : r;
      vec* p = reinterpret_cast<vec*>(reinterpret_cast<char*>(C + ro * d.ldc) + loff);
      if (d.accumulate) acc += have_old ? old : *p;
      *p = acc;
    }
    acc = 0.f;
    r = next_row(r, has_empty, rowptr, d.m);
  };
  // Accumulating calls (the per-stage sums of Alg. 2) read the old row of C at every row end.
  // With short rows that read would sit on the critical path once per row, so the rows that
  // end inside a batch are fetched together with the batch's rows of B.  (Rows are consecutive
  // in the row list unless empty rows are being stepped over.)
  // (AHEAD is chosen by the launcher for accumulating calls that walk a row list without empty rows.)
  const bool ahead = AHEAD && d.accumulate != 0 && !has_empty;

  // entry e of the chunk, clamped so that the (only) partial chunk never reads past nnz
  auto fetch = [&](int32_t e, int32_t (&c)[U], float (&v)[U]) {
    if (e + U <= e1) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        c[u] = colidx[e + u];
        v[u] = val[e + u];
      }
    } else {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int32_t ee = (e + u < e1) ? e + u : e1 - 1;
        c[u] = colidx[ee];
        v[u] = (e + u < e1) ? val[ee] : 0.f;
      }
    }
  };

  int32_t c[U];
  float v[U];
  fetch(e0, c, v);
  for (int b = 0; b < kT / U; ++b) {
    const int32_t e = e0 + b * U;
    if (e >= e1) break;
    const uint32_t fbits = (fl[(b * U) >> 5] >> ((b * U) & 31)) & (uint32_t)((1ull << U) - 1ull);
    vec h[U];
    float vc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t cc = (uint32_t)c[u] > d.kmax ? d.kmax : (uint32_t)c[u];
      h[u] = load_row<FPL, BUF>(rs, B, cc, loff, d.row_bytes, d.ldb);
      vc[u] = v[u];
    }
    vec cold[AHEAD ? U : 1];
#pragma unroll
    for (int u = 0; u < (AHEAD ? U : 1); ++u) cold[u] = 0.f;
    if (AHEAD && ahead && fbits) {
      int rr = r;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if ((fbits >> u) & 1u) {
          const int rc = rr < d.m ? rr : (int)(d.m - 1);
          const int64_t ro = rowmap ? rowmap[rc] : rc;
          cold[AHEAD ? u : 0] =
              *reinterpret_cast<const vec*>(reinterpret_cast<const char*>(C + ro * d.ldc) + loff);
          ++rr;
        }
      }
    }
    if (e + U < e1) fetch(e + U, c, v);
    // keep the U loads above together (the compiler would otherwise sink each one next to its use)
#pragma unroll
    for (int u = 0; u < U; ++u) asm volatile("" : "+v"(h[u]));
#pragma unroll
    for (int u = 0; u < U; ++u) {
      acc += vc[u] * h[u];
      if ((fbits >> u) & 1u) flush(cold[AHEAD ? u : 0], ahead);
    }
  }
  const int32_t last = e1 - 1;
  const bool closed = (flags[last >> 5] >> (last & 31)) & 1u;
  if (!closed) flush(vec(0.f), false);  // the row continues in the next chunk: store the partial sum
}

// ------------------------------------------------------------------------------------------
// narrow kernel: f <= 64 (G lanes x float4 per entry, P = 64/G entries per step)
typedef float vec4 __attribute__((ext_vector_type(4)));

template <int G>
__device__ __forceinline__ vec4 group_sum(vec4 t) {
#pragma unroll
  for (int dlt = G; dlt < 64; dlt <<= 1) {
    t.x += __shfl_xor(t.x, dlt, 64);
    t.y += __shfl_xor(t.y, dlt, 64);
    t.z += __shfl_xor(t.z, dlt, 64);
    t.w += __shfl_xor(t.w, dlt, 64);
  }
  return t;
}

template <int G, int U>
__global__ __launch_bounds__(kBlock) void spmm_narrow_kernel(SPMM_PTR_PARAMS, const SpmmDims d) {
  constexpr int P = 64 / G;
  static_assert(P <= 32 && P >= 1, "group size");
  const int lane = threadIdx.x & 63;
  const int g = lane / G, li = lane % G;
  const bool active = li * 4 < d.f;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int64_t k = (int64_t)blockIdx.x * kWavesPerBlock + wave;
  if (k >= d.nchunks) return;
  if (!ws_matches(hdr, d)) return;
  const bool has_empty = hdr->has_empty_rows != 0 && rowmap == nullptr;
  const int32_t e0 = (int32_t)(k * kT);
  const int32_t e1 = (int32_t)((d.nnz - e0 < kT) ? d.nnz : e0 + kT);
  int r = chunk_row[k];
  r = r < 0 ? 0 : (r > d.m - 1 ? (int)(d.m - 1) : r);
  bool head = rowptr[r] < e0;
  const float* __restrict__ Bl = B + li * 4;
  float* __restrict__ Cl = C + li * 4;
  float* __restrict__ carry = carry_base + k * d.carry_ld + li * 4;
  vec4 acc = 0.f;

  auto emit = [&](vec4 t) {  // t: this lane's contribution to the row that ends / is cut here
    t = group_sum<G>(t);
    if (r >= d.m) return;  // cannot happen with a consistent rowptr; keeps stores in bounds
    if (head) {
      if (g == 0 && active) *reinterpret_cast<vec4*>(carry) = t;
      head = false;
    } else if (g == 0 && active) {
      const int64_t ro = rowmap ? rowmap[r] : r;
      vec4* p = reinterpret_cast<vec4*>(Cl + ro * d.ldc);
      if (d.accumulate) t += *p;
      *p = t;
    }
    r = next_row(r, has_empty, rowptr, d.m);
  };

  constexpr int kSteps = kT / P;
  for (int s0 = 0; s0 < kSteps; s0 += U) {
    if (e0 + s0 * P >= e1) break;
    // the batch's U*P (<= 64) column ids and values arrive with one coalesced load each (lane l
    // takes the l-th entry of the batch); a step's group then picks its entry with a lane
    // permute, which keeps the vector-memory pipeline for the gathers of B
    static_assert(U * P <= 64, "a batch must fit one wavefront-wide load");
    const int32_t mine = e0 + s0 * P + lane;
    const bool have = lane < U * P && mine < e1;
    const int32_t cb = have ? colidx[mine] : 0;
    const float vb = have ? val[mine] : 0.f;
    int32_t c[U];
    float v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      c[u] = __shfl(cb, u * P + g, 64);
      v[u] = __shfl(vb, u * P + g, 64);
    }
    vec4 h[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t cc = (uint32_t)c[u] > d.kmax ? d.kmax : (uint32_t)c[u];
      h[u] = 0.f;
      if (active) h[u] = *reinterpret_cast<const vec4*>(Bl + (int64_t)cc * d.ldb);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) asm volatile("" : "+v"(h[u]));
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int32_t es = e0 + (s0 + u) * P;  // uniform
      if (es < e1) {
        uint32_t fm = (flags[es >> 5] >> (es & 31)) & (uint32_t)((1ull << P) - 1ull);
        const vec4 prod = v[u] * h[u];
        if (fm == 0) {
          acc += prod;
        } else {
          int lo = 0;
          while (fm) {
            const int j = __builtin_ctz(fm);
            fm &= fm - 1;
            vec4 t = acc;
            if (g >= lo && g <= j) t += prod;
            emit(t);
            acc = 0.f;
            lo = j + 1;
          }
          if (g >= lo) acc = prod;
        }
      }
    }
  }
  const int32_t last = e1 - 1;
  const bool closed = (flags[last >> 5] >> (last & 31)) & 1u;
  if (!closed) emit(acc);
}

// ------------------------------------------------------------------------------------------
// carries: chunk k holds a carry iff its first row began before the chunk.  The first such
// chunk of a row ("leader") sums the carries of all following chunks of the same row in a
// fixed order and adds them to C.
__global__ __launch_bounds__(kBlock) void spmm_fixup_kernel(SPMM_PTR_PARAMS, const SpmmDims d,
                                                            int32_t f_total) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int64_t k = (int64_t)blockIdx.x * kWavesPerBlock + wave;
  if (k >= d.nchunks || k == 0) return;
  if (!ws_matches(hdr, d)) return;
  int R = chunk_row[k];
  if (R < 0 || R >= d.m) return;
  const int64_t begin = rowptr[R];
  if (begin >= k * kT) return;               // no carry in this chunk
  if (begin < (k - 1) * kT) return;          // an earlier chunk leads this row
  int64_t kend = k + 1;
  while (kend < d.nchunks && chunk_row[kend] == R) ++kend;
  for (int c4 = lane; c4 * 4 < f_total; c4 += 64) {
    float4 s0 = make_float4(0.f, 0.f, 0.f, 0.f), s1 = s0, s2 = s0, s3 = s0;
    int64_t j = k;
    for (; j + 4 <= kend; j += 4) {
      const float4 t0 = *reinterpret_cast<const float4*>(carry_base + (j + 0) * d.carry_ld + c4 * 4);
      const float4 t1 = *reinterpret_cast<const float4*>(carry_base + (j + 1) * d.carry_ld + c4 * 4);
      const float4 t2 = *reinterpret_cast<const float4*>(carry_base + (j + 2) * d.carry_ld + c4 * 4);
      const float4 t3 = *reinterpret_cast<const float4*>(carry_base + (j + 3) * d.carry_ld + c4 * 4);
      s0.x += t0.x; s0.y += t0.y; s0.z += t0.z; s0.w += t0.w;
      s1.x += t1.x; s1.y += t1.y; s1.z += t1.z; s1.w += t1.w;
      s2.x += t2.x; s2.y += t2.y; s2.z += t2.z; s2.w += t2.w;
      s3.x += t3.x; s3.y += t3.y; s3.z += t3.z; s3.w += t3.w;
    }
    for (; j < kend; ++j) {
      const float4 t0 = *reinterpret_cast<const float4*>(carry_base + j * d.carry_ld + c4 * 4);
      s0.x += t0.x; s0.y += t0.y; s0.z += t0.z; s0.w += t0.w;
    }
    const int64_t ro = rowmap ? rowmap[R] : R;
    float4* p = reinterpret_cast<float4*>(C + ro * d.ldc + c4 * 4);
    float4 o = *p;
    o.x += (s0.x + s1.x) + (s2.x + s3.x);
    o.y += (s0.y + s1.y) + (s2.y + s3.y);
    o.z += (s0.z + s1.z) + (s2.z + s3.z);
    o.w += (s0.w + s1.w) + (s2.w + s3.w);
    *p = o;
  }
}

// rows without entries: C[r,:] = 0 when overwriting (no chunk ever visits them)
__global__ __launch_bounds__(kBlock) void spmm_zero_empty_kernel(SPMM_PTR_PARAMS, const SpmmDims d,
                                                                 int32_t f_total) {
  if (hdr->magic != kSpmmMagic || hdr->generation != d.generation || hdr->has_empty_rows == 0) return;
  const int lane = threadIdx.x & 63;
  const int64_t wave0 = ((int64_t)blockIdx.x * kBlock + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * kBlock) >> 6;
  for (int64_t r = wave0; r < d.m; r += nwaves) {
    if (rowptr[r + 1] != rowptr[r]) continue;
    for (int c4 = lane; c4 * 4 < f_total; c4 += 64)
      *reinterpret_cast<float4*>(C + r * d.ldc + c4 * 4) = make_float4(0.f, 0.f, 0.f, 0.f);
  }
}

// ------------------------------------------------------------------------------------------
// fallback without a prepared workspace: one wavefront per row, float4 pieces along f
__global__ __launch_bounds__(kBlock) void spmm_row_kernel(SPMM_PTR_PARAMS, const SpmmDims d,
                                                          int32_t f_total) {
  const int lane = threadIdx.x & 63;
  const int64_t wave0 = ((int64_t)blockIdx.x * kBlock + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * kBlock) >> 6;
  for (int64_t r = wave0; r < d.m; r += nwaves) {
    int32_t lo = rowptr[r], hi = rowptr[r + 1];
    lo = lo < 0 ? 0 : lo;
    hi = hi > d.nnz ? (int32_t)d.nnz : hi;
    for (int c4 = lane; c4 * 4 < f_total; c4 += 64) {
      // two-level sum: runs of 128 entries, then the runs (keeps the rounding error of a long
      // row of equal terms from growing with the row length)
      float4 acc = make_float4(0.f, 0.f, 0.f, 0.f), tot = acc;
      for (int32_t e = lo; e < hi; ++e) {
        const uint32_t c = (uint32_t)colidx[e];
        const uint32_t cc = c > d.kmax ? d.kmax : c;
        const float v = val[e];
        const float4 h = *reinterpret_cast<const float4*>(B + (int64_t)cc * d.ldb + c4 * 4);
        acc.x += v * h.x; acc.y += v * h.y; acc.z += v * h.z; acc.w += v * h.w;
        if (((e - lo) & 127) == 127) {
          tot.x += acc.x; tot.y += acc.y; tot.z += acc.z; tot.w += acc.w;
          acc = make_float4(0.f, 0.f, 0.f, 0.f);
        }
      }
      acc.x += tot.x; acc.y += tot.y; acc.z += tot.z; acc.w += tot.w;
      float4* p = reinterpret_cast<float4*>(C + r * d.ldc + c4 * 4);
      if (d.accumulate) {
        const float4 o = *p;
        acc.x += o.x; acc.y += o.y; acc.z += o.z; acc.w += o.w;
      }
      *p = acc;
    }
  }
}

// ------------------------------------------------------------------------------------------
// preparation
__global__ __launch_bounds__(kBlock) void prep_clear_flags_kernel(uint32_t* flags, int64_t words) {
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < words; i += stride) flags[i] = 0;
}

// chunk_row[k] = last row r with rowptr[r] <= k*kT (the non-empty row that holds entry k*kT)
__global__ __launch_bounds__(kBlock) void prep_chunks_kernel(const int32_t* __restrict__ rowptr,
                                                             int64_t m, int64_t nchunks,
                                                             int32_t* __restrict__ chunk_row) {
  const int64_t k = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (k > nchunks) return;
  if (k == nchunks) {
    chunk_row[k] = (int32_t)m;
    return;
  }
  const int64_t target = k * kT;
  int64_t lo = 0, hi = m;  // invariant: rowptr[lo] <= target; answer in [lo, hi)
  while (hi - lo > 1) {
    const int64_t mid = (lo + hi) >> 1;
    if ((int64_t)rowptr[mid] <= target) lo = mid; else hi = mid;
  }
  chunk_row[k] = (int32_t)lo;
}

__global__ __launch_bounds__(kBlock) void prep_rowend_kernel(const int32_t* __restrict__ rowptr,
                                                             int64_t m, int64_t nnz,
                                                             uint32_t* __restrict__ flags,
                                                             int32_t* __restrict__ has_empty) {
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  for (int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x; r < m; r += stride) {
    const int64_t b = rowptr[r], e = rowptr[r + 1];
    if (e > b && e <= nnz && e >= 1) {
      atomicOr(&flags[(e - 1) >> 5], 1u << ((e - 1) & 31));
    } else if (e == b) {
      *has_empty = 1;
    }
  }
}

inline unsigned capped_grid(int64_t blocks) {
  const int64_t cap = 256 * 64;
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  return (unsigned)blocks;
}

struct SpmmPtrs {
  const int32_t* rowptr; const int32_t* colidx; const float* val; const float* B; float* C;
  const SpmmWsHeader* hdr; const int32_t* chunk_row; const uint32_t* flags; float* carry;
  const int32_t* rowmap;
};

template <typename Kern, typename... Extra>
inline void launch_waves(Kern kern, int64_t blocks, const SpmmPtrs& p, const SpmmDims& d,
                         hipStream_t s, Extra... extra) {
  hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(kBlock), 0, s, p.rowptr, p.colidx, p.val,
                     p.B, p.C, p.hdr, p.chunk_row, p.flags, p.carry, p.rowmap, d, extra...);
}

// chunk-table construction for a CSR (rowptr of `rows` rows, `nnz` entries)
int build_chunk_tables(const int32_t* d_rowptr, int64_t rows, int64_t nnz, int32_t* chunk_row,
                       uint32_t* flags, int32_t* d_has_empty, hipStream_t s) {
  const int64_t nchunks = spmm_nchunks(nnz);
  const int64_t words = nchunks * (kSpmmChunk / 32);
  if (words > 0) {
    hipLaunchKernelGGL(prep_clear_flags_kernel, dim3(capped_grid(ceil_div(words, kBlock))), dim3(kBlock),
                       0, s, flags, words);
    SAGNN_LAUNCH_CHECK();
  }
  if (rows > 0) {
    hipLaunchKernelGGL(prep_chunks_kernel, dim3((unsigned)ceil_div(nchunks + 1, kBlock)), dim3(kBlock), 0,
                       s, d_rowptr, rows, nchunks, chunk_row);
    SAGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(prep_rowend_kernel, dim3(capped_grid(ceil_div(rows, kBlock))), dim3(kBlock), 0, s,
                       d_rowptr, rows, nnz, flags, d_has_empty);
    SAGNN_LAUNCH_CHECK();
  }
  return SAGNN_OK;
}

}  // namespace

uint64_t spmm_next_generation();
int sweep_combine(const SpmmHostDesc& d, const SpmmWsLayout& L, char* ws, float* C, int64_t ldc,
                  int32_t f_total, int32_t accumulate, hipStream_t s);

namespace {
int launch_spmm_body(const int32_t* rowptr, const int32_t* colidx, const float* val, int64_t m,
                     int64_t k, int64_t nnz, const float* B, int64_t ldb, int32_t f, float* C,
                     int64_t ldc, int32_t accumulate, void* ws, size_t ws_bytes, hipStream_t s, bool inner);
}
int launch_spmm(const int32_t* rowptr, const int32_t* colidx, const float* val, int64_t m,
                int64_t k, int64_t nnz, const float* B, int64_t ldb, int32_t f, float* C,
                int64_t ldc, int32_t accumulate, void* ws, size_t ws_bytes, hipStream_t s) {
  return launch_spmm_body(rowptr, colidx, val, m, k, nnz, B, ldb, f, C, ldc, accumulate, ws, ws_bytes, s, false);
}
namespace {
// inner: the call is the rest-CSR part of a workspace prepared with dense tiles
int launch_spmm_body(const int32_t* rowptr, const int32_t* colidx, const float* val, int64_t m,
                     int64_t k, int64_t nnz, const float* B, int64_t ldb, int32_t f, float* C,
                     int64_t ldc, int32_t accumulate, void* ws, size_t ws_bytes, hipStream_t s, bool inner) {
  if (m < 0 || k < 0 || nnz < 0 || f <= 0 || (f & 3) || ldb < f || ldc < f || (ldb & 3) ||
      (ldc & 3) || m > 0x7FFFFFFFll || k > 0x7FFFFFFFll || nnz > 0x7FFFFFFFll)
    return SAGNN_EINVAL;
  if (accumulate != 0 && accumulate != 1) return SAGNN_EINVAL;
  if (m == 0) return SAGNN_OK;
  if (!rowptr || !C || !aligned16(C)) return SAGNN_EINVAL;
  if (nnz > 0 && (!colidx || !val || !B || !aligned16(B) || k == 0)) return SAGNN_EINVAL;
  if (ws && (reinterpret_cast<uintptr_t>(ws) & 255u)) return SAGNN_EINVAL;

  SpmmPtrs p{};
  p.rowptr = rowptr; p.colidx = colidx; p.val = val; p.B = B; p.C = C;
  SpmmDims d{};
  d.m = m; d.nnz = nnz; d.ldb = ldb; d.ldc = ldc;
  d.kmax = k > 0 ? (uint32_t)(k - 1) : 0u;
  d.f = f; d.accumulate = accumulate;
  d.nchunks = spmm_nchunks(nnz);
  d.carry_ld = f;

  if (!ws) {
    launch_waves(spmm_row_kernel, capped_grid(ceil_div(m, kWavesPerBlock)), p, d, s, f);
    SAGNN_LAUNCH_CHECK();
    return SAGNN_OK;
  }

  SpmmHostDesc desc{};
  if (!spmm_desc_get(ws, &desc)) return SAGNN_EINVAL;        // never prepared in this process
  if (desc.tiles && !inner) {
    // dense tiles: the rest CSR (stored behind the plain workspace) through the schedule prepared
    // for it, then C += tiles * B out of LDS
    if (desc.m != m || desc.full_nnz != nnz || desc.f != f || k < desc.k) return SAGNN_EINVAL;
    const size_t plain = round_up(spmm_ws_bytes(m, desc.full_nnz, desc.f), 256);
    const TileWsLayout TL = tile_ws_layout(m, desc.k, desc.full_nnz, desc.f);
    if (ws_bytes < plain + TL.total) return SAGNN_ECAPACITY;
    char* tb = reinterpret_cast<char*>(ws) + plain;
    int rc = launch_spmm_body(reinterpret_cast<const int32_t*>(tb + TL.rest_rowptr),
                              reinterpret_cast<const int32_t*>(tb + TL.rest_col),
                              reinterpret_cast<const float*>(tb + TL.rest_val), m, k, desc.nnz, B, ldb, f, C, ldc,
                              accumulate, ws, plain, s, true);
    if (rc != SAGNN_OK) return rc;
    TilePlan tp{};
    tp.n_ts = desc.tile_count; tp.n_items = desc.tile_items; tp.entries = desc.tile_entries;
    tp.rest_nnz = desc.nnz; tp.rows = desc.tile_rows;
    return tile_launch(tp, desc.tile_generation, tb, TL, B, ldb, d.kmax, f, m, C, ldc, s);
  }
  if (desc.m != m || desc.nnz != nnz || desc.f < f) return SAGNN_EINVAL;
  // the re-ordered entry streams hold column ids checked against the k of the preparation: an
  // operand with fewer rows would be read out of range
  if (nnz > 0 && k < desc.k) return SAGNN_EINVAL;
  const SpmmWsLayout L = spmm_ws_layout(m, nnz, desc.f);
  if (ws_bytes < L.total) return SAGNN_ECAPACITY;
  char* base = reinterpret_cast<char*>(ws);
  p.hdr = reinterpret_cast<const SpmmWsHeader*>(base + L.header);
  p.chunk_row = reinterpret_cast<const int32_t*>(base + L.chunk_row);
  p.flags = reinterpret_cast<const uint32_t*>(base + L.flags);
  p.carry = reinterpret_cast<float*>(base + L.carry);
  d.generation = desc.generation;

  if (!accumulate && desc.has_empty_rows) {
    launch_waves(spmm_zero_empty_kernel, capped_grid(ceil_div(m, kWavesPerBlock)), p, d, s, f);
    SAGNN_LAUNCH_CHECK();
  }
  if (desc.mode == 1) {
    // the sweep schedule exists for multiples of 64 and, in grouped form, for exactly 32 and 16
    if ((f & 63) && !((f == 32 || f == 16) && f == desc.f)) return SAGNN_EINVAL;
    if (desc.groups >= 8 && f != desc.f) return SAGNN_EINVAL;
    // the chunk kernels walk the compacted short-row CSR stored in the workspace
    const int64_t short_base = (int64_t)round_up((size_t)desc.sweep_stream_len + 64, 256);
    p.rowptr = reinterpret_cast<const int32_t*>(base + L.rowptr_s);
    p.rowmap = reinterpret_cast<const int32_t*>(base + L.rowmap_s);
    p.colidx = reinterpret_cast<const int32_t*>(base + L.code) + short_base;
    p.val = reinterpret_cast<const float*>(base + L.vals) + short_base;
    d.m = desc.c_rows; d.nnz = desc.c_nnz; d.nchunks = desc.c_nchunks;
  } else if (desc.c_rows != m) {
    // empty rows were taken out of the row list when the workspace was prepared
    p.rowptr = reinterpret_cast<const int32_t*>(base + L.rowptr_s);
    p.rowmap = reinterpret_cast<const int32_t*>(base + L.rowmap_s);
    d.m = desc.c_rows;
  }

  const int64_t blocks = ceil_div(d.nchunks, kWavesPerBlock);
  const int32_t max_slab = desc.mode == 1 && desc.max_slab == 128 ? 128 : 256;
  // column slabs: 256 / 128 / 64 wide through the wide kernels, the rest through the narrow one
  int32_t col0 = 0;
  while (col0 < f) {
    const int32_t rest = f - col0;
    SpmmPtrs sp = p;
    SpmmDims sd = d;
    sp.B = B + col0; sp.C = C + col0; sp.carry = p.carry + col0;
    sd.f = rest >= 256 && max_slab >= 256 ? 256 : (rest >= 128 ? 128 : (rest >= 64 ? 64 : rest));
    const bool buf = buffer_addressable(d.kmax, ldb, sd.f, &sd.b_bytes);
    sd.row_bytes = (uint32_t)(ldb * 4);
    if (desc.mode == 1) {
      int rc = sweep_launch(desc, L, base, B, ldb, col0, sd.f, d.kmax, C, ldc, accumulate, f, s);
      if (rc != SAGNN_OK) return rc;
    }
    if (d.nchunks > 0) {
      // accumulating calls over a row list without empty rows fetch the old rows of C ahead
      const bool ahead = accumulate != 0 && !(desc.has_empty_rows && sp.rowmap == nullptr);
#define SAGNN_WIDE(FPL_, BUF_)                                                              \
  (ahead ? launch_waves(spmm_wide_kernel<FPL_, 8, BUF_, true>, blocks, sp, sd, s)           \
         : launch_waves(spmm_wide_kernel<FPL_, 8, BUF_, false>, blocks, sp, sd, s))
      if (sd.f == 256 && buf) SAGNN_WIDE(4, true);
      else if (sd.f == 256) SAGNN_WIDE(4, false);
      else if (sd.f == 128 && buf) SAGNN_WIDE(2, true);
      else if (sd.f == 128) SAGNN_WIDE(2, false);
      else if (sd.f == 64 && buf) SAGNN_WIDE(1, true);
      else if (sd.f == 64) SAGNN_WIDE(1, false);
#undef SAGNN_WIDE
      else if (rest > 32) launch_waves(spmm_narrow_kernel<16, 4>, blocks, sp, sd, s);
      else if (rest > 16) launch_waves(spmm_narrow_kernel<8, 4>, blocks, sp, sd, s);
      else if (rest > 8) launch_waves(spmm_narrow_kernel<4, 4>, blocks, sp, sd, s);
      else launch_waves(spmm_narrow_kernel<2, 2>, blocks, sp, sd, s);
      SAGNN_LAUNCH_CHECK();
    }
    col0 += sd.f;
  }
  if (d.nchunks > 1) {
    launch_waves(spmm_fixup_kernel, blocks, p, d, s, f);
    SAGNN_LAUNCH_CHECK();
  }
  if (desc.mode == 1) {
    int rc = sweep_combine(desc, L, base, C, ldc, f, accumulate, s);
    if (rc != SAGNN_OK) return rc;
  }
  return SAGNN_OK;
}
}  // namespace

// ------------------------------------------------------------------------------------------
// The layer with the dense transform as the epilogue of the slab sweep (spmm_sweep_fused_kernel)
// covers the rows that one wavefront of the sweep finishes.  The others -- rows outside the sweep
// (short rows) and rows cut into several pieces -- are few where this form is used and go
// through this kernel: one wavefront per row computes the row of T (a gather over the row's
// entries, or the sum of the row's partial rows in a fixed order), puts it into LDS and
// multiplies it by W, 64 output columns at a time.
namespace {
constexpr int64_t kFusedLeftoverMax = 65536;   // rows; above that the row-range kernel serves the layer

template <int FPL, bool BF16>
__global__ __launch_bounds__(256) void layer_leftover_kernel(
    const int32_t* __restrict__ rowptr_s, const int32_t* __restrict__ rowmap_s,
    const int32_t* __restrict__ colidx_s, const float* __restrict__ val_s, int64_t n_short, int64_t nnz_s,
    const int32_t* __restrict__ multi_row, const int32_t* __restrict__ multi_first, int64_t n_multi,
    const float* __restrict__ partial, const SpmmWsHeader* __restrict__ hdr, uint64_t generation,
    const float* __restrict__ B, int64_t ldb, uint32_t kmax, const SweepFusedArgs fa) {
  using vec = typename Vec<FPL>::T;
  constexpr int kRow = 64 * FPL;
  __shared__ float trow[4][kRow];
  if (hdr->magic != kSpmmMagic || hdr->generation != generation) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t i = (int64_t)blockIdx.x * 4 + wave;
  int64_t row = -1;
  vec t = 0.f;
  if (i < n_short) {
    row = rowmap_s[i];
    int32_t b = rowptr_s[i], e = rowptr_s[i + 1];
    b = b < 0 ? 0 : b;
    e = e > nnz_s ? (int32_t)nnz_s : e;
    for (int32_t q = b; q < e; ++q) {
      const uint32_t cc = (uint32_t)colidx_s[q];
      const uint32_t c = cc > kmax ? kmax : cc;
      t += val_s[q] * *reinterpret_cast<const vec*>(B + (int64_t)c * ldb + lane * FPL);
    }
  } else if (i < n_short + n_multi) {
    const int64_t q = i - n_short;
    row = multi_row[q];
    for (int32_t j = multi_first[q]; j < multi_first[q + 1]; ++j)
      t += *reinterpret_cast<const vec*>(partial + (int64_t)j * kRow + lane * FPL);
  }
  if (row >= 0 && fa.T) *reinterpret_cast<vec*>(fa.T + row * kRow + lane * FPL) = t;
  if constexpr (FPL == 1) {
    trow[wave][lane] = BF16 ? (float)(__bf16)t : t;
  } else {
#pragma unroll
    for (int c = 0; c < FPL; ++c) trow[wave][lane * FPL + c] = BF16 ? (float)(__bf16)t[c] : t[c];
  }
  __syncthreads();
  if (row < 0) return;
  for (int col = lane; col < fa.f_out; col += 64) {
    float z = 0.f;
    for (int k = 0; k < kRow; ++k) {
      const float w = fa.W[(int64_t)k * fa.f_out + col];
      z += trow[wave][k] * (BF16 ? (float)(__bf16)w : w);
    }
    if (fa.Z) fa.Z[row * fa.f_out + col] = z;
    if (fa.Hout) fa.Hout[row * fa.f_out + col] = fa.act == SAGNN_ACT_RELU ? (z > 0.f ? z : 0.f) : z;
  }
}
}  // namespace

bool fused_sweep_layer_applicable(const void* ws, int32_t f_in, int32_t f_out) {
  SpmmHostDesc desc{};
  if (!ws || !spmm_desc_get(ws, &desc)) return false;
  if (desc.tiles) return false;   // rows with entries in dense tiles are not finished by the sweep
  if (desc.mode != 1 || desc.slots != kSweepSlots || desc.n_waves <= 0 || (desc.n_waves & 3)) return false;
  if (!(f_in == 64 || f_in == 128 || f_in == 256) || f_in > desc.f || f_in > desc.max_slab) return false;
  // the launch must cover the whole width of T with one kernel of the prepared schedule
  if (desc.groups == 2 ? f_in > 128 : (desc.groups == 4 ? f_in != 64 : desc.groups != 1)) return false;
  if (f_out <= 0 || (f_out & 3) || f_out > 256) return false;
  return desc.c_rows + desc.n_multi_rows <= kFusedLeftoverMax;
}

int launch_fused_sweep_layer(const int32_t* rowptr, const int32_t* colidx, const float* val, int64_t m,
                             int64_t k, int64_t nnz, const float* H, int64_t ldh, int32_t f_in,
                             const float* W, int32_t f_out, int32_t act, int32_t prec, float* T, float* Z,
                             float* Hout, void* ws, size_t ws_bytes, hipStream_t s) {
  (void)colidx; (void)val;   // the prepared workspace holds its own copy of the entries
  SpmmHostDesc desc{};
  if (!fused_sweep_layer_applicable(ws, f_in, f_out) || !spmm_desc_get(ws, &desc)) return 1;
  if (desc.m != m || desc.nnz != nnz) return SAGNN_EINVAL;
  if (prec != SAGNN_GEMM_FP32 && prec != SAGNN_GEMM_BF16 && prec != SAGNN_GEMM_FP32_BF16X3) return SAGNN_EINVAL;
  if (act != SAGNN_ACT_IDENTITY && act != SAGNN_ACT_RELU) return SAGNN_EINVAL;
  if (nnz > 0 && k < desc.k) return SAGNN_EINVAL;
  if (!rowptr || !H || !W || (!Z && !Hout) || ldh < f_in || (ldh & 3) || !aligned16(H)) return SAGNN_EINVAL;
  const SpmmWsLayout L = spmm_ws_layout(m, nnz, desc.f);
  if (ws_bytes < L.total) return SAGNN_ECAPACITY;
  char* base = reinterpret_cast<char*>(ws);
  const SpmmWsHeader* hdr = reinterpret_cast<const SpmmWsHeader*>(base + L.header);
  const uint32_t kmax = k > 0 ? (uint32_t)(k - 1) : 0u;
  const bool bf16 = prec == SAGNN_GEMM_BF16;   // (the few rows left to the small kernel: three-term mode uses fp32 there)

  if (desc.has_empty_rows) {   // a row without entries: T = 0, so Z = 0 and sigma(0) = 0
    SpmmPtrs p{};
    p.rowptr = rowptr; p.hdr = hdr;
    SpmmDims d{};
    d.m = m; d.generation = desc.generation;
    float* outs[3] = {Z, Hout, T};
    const int32_t widths[3] = {f_out, f_out, f_in};
    for (int o = 0; o < 3; ++o) {
      if (!outs[o]) continue;
      p.C = outs[o];
      d.ldc = widths[o];
      launch_waves(spmm_zero_empty_kernel, capped_grid(ceil_div(m, kWavesPerBlock)), p, d, s, widths[o]);
      SAGNN_LAUNCH_CHECK();
    }
  }
  SweepFusedArgs fa{};
  fa.W = W; fa.Z = Z; fa.Hout = Hout; fa.T = T; fa.f_out = f_out; fa.act = act;
  int rc = sweep_launch_fused(desc, L, base, H, ldh, f_in, kmax, fa, prec, s);   // (operand modes are numbered like prec)
  if (rc != SAGNN_OK) return rc;
  const int64_t left = desc.c_rows + desc.n_multi_rows;
  if (left > 0) {
    const int64_t short_base = (int64_t)round_up((size_t)desc.sweep_stream_len + 64, 256);
    auto go = [&](auto kern) -> int {
      hipLaunchKernelGGL(kern, dim3((unsigned)ceil_div(left, 4)), dim3(256), 0, s,
                         reinterpret_cast<const int32_t*>(base + L.rowptr_s),
                         reinterpret_cast<const int32_t*>(base + L.rowmap_s),
                         reinterpret_cast<const int32_t*>(base + L.code) + short_base,
                         reinterpret_cast<const float*>(base + L.vals) + short_base, desc.c_rows, desc.c_nnz,
                         reinterpret_cast<const int32_t*>(base + L.multi_row),
                         reinterpret_cast<const int32_t*>(base + L.multi_first), desc.n_multi_rows,
                         reinterpret_cast<const float*>(base + L.partial), hdr, desc.generation, H, ldh, kmax, fa);
      SAGNN_LAUNCH_CHECK();
      return SAGNN_OK;
    };
    if (f_in == 256) rc = bf16 ? go(layer_leftover_kernel<4, true>) : go(layer_leftover_kernel<4, false>);
    else if (f_in == 128) rc = bf16 ? go(layer_leftover_kernel<2, true>) : go(layer_leftover_kernel<2, false>);
    else rc = bf16 ? go(layer_leftover_kernel<1, true>) : go(layer_leftover_kernel<1, false>);
    if (rc != SAGNN_OK) return rc;
  }
  return SAGNN_OK;
}

}  // namespace sagnn

SAGNN_EXPORT int spmm_csr_workspace_bytes(int64_t m, int64_t nnz, int32_t f, size_t* bytes) {
  using namespace sagnn;
  if (!bytes || m < 0 || nnz < 0 || f <= 0 || (f & 3) || nnz > 0x7FFFFFFFll || m > 0x7FFFFFFFll)
    return SAGNN_EINVAL;
  *bytes = spmm_ws_bytes(m, nnz, f);
  return SAGNN_OK;
}

SAGNN_EXPORT int spmm_csr_workspace_bytes_opt(int64_t m, int64_t k, int64_t nnz, int32_t f,
                                              const sagnn_spmm_options* h_opt, size_t* bytes) {
  using namespace sagnn;
  if (!bytes || m < 0 || k < 0 || nnz < 0 || f <= 0 || (f & 3) || nnz > 0x7FFFFFFFll || m > 0x7FFFFFFFll ||
      k > 0x7FFFFFFFll)
    return SAGNN_EINVAL;
  size_t b = spmm_ws_bytes(m, nnz, f);
  TileGeom g{};
  if (h_opt && h_opt->dense_tiles == 1 && tile_geom(f, &g)) b = round_up(b, 256) + tile_ws_layout(m, k, nnz, f).total;
  *bytes = b;
  return SAGNN_OK;
}

SAGNN_EXPORT int spmm_csr_tile_info(const void* d_ws, int64_t* h_info) {
  using namespace sagnn;
  if (!d_ws || !h_info) return SAGNN_EINVAL;
  SpmmHostDesc d{};
  if (!spmm_desc_get(d_ws, &d)) return SAGNN_EINVAL;
  h_info[0] = d.tiles;
  h_info[1] = d.tiles ? d.tile_entries : 0;
  h_info[2] = d.tiles ? d.tile_count : 0;
  h_info[3] = d.tiles ? d.tile_items : 0;
  h_info[4] = d.tiles ? d.tile_rows : 0;
  h_info[5] = d.tiles ? d.nnz : 0;
  return SAGNN_OK;
}

SAGNN_EXPORT int spmm_csr_prepare_opt(const int32_t* d_rowptr, const int32_t* d_colidx,
                                      const float* d_val, int64_t m, int64_t k, int64_t nnz, int32_t f,
                                      void* d_ws, size_t ws_bytes, const sagnn_spmm_options* h_opt,
                                      void* stream) {
  using namespace sagnn;
  sagnn_spmm_options opt{};
  if (h_opt) opt = *h_opt;
  if (opt.short_rows < -1 || opt.short_rows > 1 ||
      (opt.slab_width != 0 && opt.slab_width != 128 && opt.slab_width != 256))
    return SAGNN_EINVAL;
  if (m < 0 || k < 0 || nnz < 0 || f <= 0 || (f & 3) || m > 0x7FFFFFFFll || nnz > 0x7FFFFFFFll ||
      k > 0x7FFFFFFFll)
    return SAGNN_EINVAL;
  if (!d_rowptr || !d_ws || (reinterpret_cast<uintptr_t>(d_ws) & 255u)) return SAGNN_EINVAL;
  if (nnz > 0 && (!d_colidx || !d_val)) return SAGNN_EINVAL;
  const SpmmWsLayout L = spmm_ws_layout(m, nnz, f);
  if (ws_bytes < L.total) return SAGNN_ECAPACITY;
  hipStream_t s = (hipStream_t)stream;
  char* base = reinterpret_cast<char*>(d_ws);
  if (opt.dense_tiles < -1 || opt.dense_tiles > 1 || opt.tile_reuse_x10 < 0) return SAGNN_EINVAL;
  TileGeom tg{};
  if (opt.dense_tiles == 1 && tile_geom(f, &tg) && m > 0 && k > 0 && nnz > 0) {
    // dense tiles: split A into the kept tiles and a rest CSR (both in the tile region behind the
    // plain workspace), then prepare the rest like any other matrix
    const size_t plain = round_up(L.total, 256);
    const TileWsLayout TL = tile_ws_layout(m, k, nnz, f);
    if (ws_bytes < plain + TL.total) return SAGNN_ECAPACITY;
    TilePlan tp{};
    const uint64_t gen = spmm_next_generation();
    int rc = tile_prepare(d_rowptr, d_colidx, d_val, m, k, nnz, f, base + plain, TL, opt.tile_reuse_x10, gen, s, &tp);
    if (rc != SAGNN_OK) return rc;
    if (tp.n_ts > 0) {
      sagnn_spmm_options inner_opt = opt;
      inner_opt.dense_tiles = -1;
      char* tb = base + plain;
      rc = spmm_csr_prepare_opt(reinterpret_cast<const int32_t*>(tb + TL.rest_rowptr),
                                reinterpret_cast<const int32_t*>(tb + TL.rest_col),
                                reinterpret_cast<const float*>(tb + TL.rest_val), m, k, tp.rest_nnz, f, d_ws, plain,
                                &inner_opt, stream);
      if (rc != SAGNN_OK) return rc;
      SpmmHostDesc desc{};
      if (!spmm_desc_get(d_ws, &desc)) return SAGNN_EINVAL;
      desc.tiles = 1;
      desc.full_nnz = nnz;
      desc.tile_count = tp.n_ts; desc.tile_items = tp.n_items; desc.tile_entries = tp.entries;
      desc.tile_rows = tp.rows; desc.tile_generation = gen;
      spmm_desc_put(d_ws, desc);
      return SAGNN_OK;
    }
    // no tile is dense enough: the plain preparation below
  }
  int32_t* d_has_empty = reinterpret_cast<int32_t*>(base + L.carry);  // scratch until the first product

  SweepPlanResult plan{};
  if ((f & 63) == 0 || f == 32 || f == 16) {
    int rc = sweep_prepare(d_rowptr, d_colidx, d_val, m, k, nnz, f, base, L, opt, s, &plan);
    if (rc != SAGNN_OK) return rc;
  }
  SpmmWsHeader h{};
  SAGNN_HIP(hipMemsetAsync(d_has_empty, 0, 4, s));   // set-up call: never recorded into a graph
  if (plan.use_sweep) {
    h = plan.hdr;
    int rc = build_chunk_tables(reinterpret_cast<const int32_t*>(base + L.rowptr_s), h.c_rows, h.c_nnz,
                                reinterpret_cast<int32_t*>(base + L.chunk_row),
                                reinterpret_cast<uint32_t*>(base + L.flags), d_has_empty, s);
    if (rc != SAGNN_OK) return rc;
  } else {
    h.magic = kSpmmMagic;
    h.m = m; h.nnz = nnz; h.f = f; h.mode = 0;
    h.generation = spmm_next_generation();
    h.c_rows = m; h.c_nnz = nnz; h.c_nchunks = spmm_nchunks(nnz);
    int rc = build_chunk_tables(d_rowptr, m, nnz, reinterpret_cast<int32_t*>(base + L.chunk_row),
                                reinterpret_cast<uint32_t*>(base + L.flags), d_has_empty, s);
    if (rc != SAGNN_OK) return rc;
    int32_t he = 0;
    SAGNN_HIP(hipMemcpyAsync(&he, d_has_empty, 4, hipMemcpyDeviceToHost, s));
    SAGNN_HIP(hipStreamSynchronize(s));
    h.has_empty_rows = he;
    if (he && nnz > 0) {
      // Rows without entries (e.g. one column block of a row block, Alg. 2) would make a chunk's
      // wavefront step over them one dependent load at a time.  Walk a row list without them
      // instead: the same compacted-CSR form the short rows of the sweep schedule use.
      // The row pass of the sweep planner with a threshold no row reaches makes exactly that list
      // (every row with entries is "short").
      SweepRowTotals t{};
      rc = sweep_plan_rows(d_rowptr, m, nnz, 0x7FFFFFFF, 1024, base, L, s, &t);
      if (rc != SAGNN_OK) return rc;
      if (!t.bad && t.short_entries == nnz) {   // (a malformed row pointer keeps the plain walk, which clamps everything)
        rc = build_chunk_tables(reinterpret_cast<const int32_t*>(base + L.rowptr_s), t.short_rows, nnz,
                                reinterpret_cast<int32_t*>(base + L.chunk_row),
                                reinterpret_cast<uint32_t*>(base + L.flags), d_has_empty, s);
        if (rc != SAGNN_OK) return rc;
        h.c_rows = t.short_rows;
      }
    }
  }
  SAGNN_HIP(hipMemcpyAsync(base + L.header, &h, sizeof(h), hipMemcpyHostToDevice, s));
  SAGNN_HIP(hipStreamSynchronize(s));
  SpmmHostDesc desc{};
  desc.generation = h.generation; desc.m = m; desc.nnz = nnz; desc.f = f; desc.mode = h.mode;
  desc.c_rows = h.c_rows; desc.c_nnz = h.c_nnz; desc.c_nchunks = h.c_nchunks;
  desc.n_waves = h.n_waves; desc.n_multi_rows = h.n_multi_rows; desc.has_empty_rows = h.has_empty_rows;
  desc.sweep_stream_len = h.n_long_entries;
  desc.groups = h.groups > 0 ? h.groups : 1;
  desc.k = k;
  desc.n_intervals = h.n_intervals; desc.sync_slabs = h.sync_slabs; desc.wg_per_cohort = h.wg_per_cohort;
  desc.sync_timeout_ticks = h.sync_timeout_ticks; desc.sync_test_extra = h.sync_test_extra;
  desc.slots = h.slots;
  desc.max_slab = h.max_slab > 0 ? h.max_slab : 256;
  desc.barriers = h.barriers; desc.pace_ps_per_step = h.pace_ps_per_step > 0 ? h.pace_ps_per_step : 0;
  desc.mean_steps = plan.mean_steps;
  desc.max_steps = plan.max_steps;
  spmm_desc_put(d_ws, desc);
  return SAGNN_OK;
}

SAGNN_EXPORT int spmm_csr_prepare(const int32_t* d_rowptr, const int32_t* d_colidx,
                                  const float* d_val, int64_t m, int64_t k, int64_t nnz, int32_t f,
                                  void* d_ws, size_t ws_bytes, void* stream) {
  return spmm_csr_prepare_opt(d_rowptr, d_colidx, d_val, m, k, nnz, f, d_ws, ws_bytes, nullptr, stream);
}

SAGNN_EXPORT int spmm_csr_prepare_tuned(const int32_t* d_rowptr, const int32_t* d_colidx,
                                        const float* d_val, int64_t m, int64_t k, int64_t nnz,
                                        int32_t f, void* d_ws, size_t ws_bytes, const float* d_B,
                                        int64_t ldb, float* d_C, int64_t ldc, int32_t* h_choice,
                                        const sagnn_spmm_options* h_opt, void* stream) {
  using namespace sagnn;
  if (!d_B || !d_C || ldb < f || ldc < f) return SAGNN_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  // (piece, long-row threshold) variants of the slab-sweep plan; {0, 0} is spmm_csr_prepare's own
  struct Cand { int piece, min_long, slab; };
  static const Cand cand[] = {{0, 0, 0}, {4608, 0, 0}, {3584, 0, 0}, {0, 96, 0}, {4608, 96, 0},
                              {0, 0, 128}, {4608, 0, 128}};
  // the 128-wide-slab variants only exist for operands wider than 128
  const int n_cand = (f > 128 && (f & 63) == 0 && !(h_opt && h_opt->slab_width != 0)) ? 7 : 5;
  // a variant only replaces choices the planner would make by itself: where it picks the
  // lower long-row threshold (near-regular matrices) the candidate threshold is not forced
  auto options_of = [&](int c) {
    sagnn_spmm_options o{};
    if (h_opt) o = *h_opt;
    if (cand[c].piece > 0) o.piece = cand[c].piece;
    if (cand[c].min_long > 0) o.min_long = -cand[c].min_long;   // negative: "where you would pick 64"
    if (cand[c].slab > 0) o.slab_width = cand[c].slab;
    return o;
  };
  int best = -1, last = -1;
  float best_ms = 0.f;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  auto cleanup = [&]() {
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  };
  for (int c = 0; c < n_cand; ++c) {
    const sagnn_spmm_options o = options_of(c);
    int rc = spmm_csr_prepare_opt(d_rowptr, d_colidx, d_val, m, k, nnz, f, d_ws, ws_bytes, &o, stream);
    if (rc != SAGNN_OK) { cleanup(); return rc; }
    last = c;
    SpmmHostDesc desc{};
    if (!spmm_desc_get(d_ws, &desc) || desc.mode != 1) { best = c; break; }   // nothing to tune
    if (!e0) {
      hipError_t e = hipEventCreate(&e0);
      if (e == hipSuccess) e = hipEventCreate(&e1);
      if (e != hipSuccess) { set_hip_error(e); cleanup(); return SAGNN_EHIP; }
    }
    float ms_min = 0.f;
    for (int rep = 0; rep < 6; ++rep) {   // the first run warms the caches and is not counted
      hipError_t e = hipEventRecord(e0, s);
      if (e != hipSuccess) { set_hip_error(e); cleanup(); return SAGNN_EHIP; }
      rc = launch_spmm(d_rowptr, d_colidx, d_val, m, k, nnz, d_B, ldb, f, d_C, ldc, 0, d_ws, ws_bytes, s);
      if (rc != SAGNN_OK) { cleanup(); return rc; }
      float ms = 0.f;
      e = hipEventRecord(e1, s);
      if (e == hipSuccess) e = hipEventSynchronize(e1);
      if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
      if (e != hipSuccess) { set_hip_error(e); cleanup(); return SAGNN_EHIP; }
      if (rep == 1 || (rep > 1 && ms < ms_min)) ms_min = ms;
    }
    // a variant has to beat the default plan by more than the run-to-run noise of the timing
    if (best < 0 || ms_min < (best == 0 ? 0.985f * best_ms : best_ms)) { best = c; best_ms = ms_min; }
  }
  if (best != last) {
    const sagnn_spmm_options o = options_of(best);
    int rc = spmm_csr_prepare_opt(d_rowptr, d_colidx, d_val, m, k, nnz, f, d_ws, ws_bytes, &o, stream);
    if (rc != SAGNN_OK) { cleanup(); return rc; }
  }
  // Pacing of the sweep (see sweep_pace_until): lay the kept plan out with intervals and search
  // the time per stream step that makes the product fastest.  Upper end: the whole free-running
  // call time spread over the schedule of the generations of wavefronts; the useful values lie
  // below it, because a paced sweep misses less in L2.  Below some value the wavefronts cannot
  // keep to the schedule and the product falls back to its free-running time, so the search
  // walks down and stops there.  If pacing does not pay, the plain layout is restored.
  {
    SpmmHostDesc desc{};
    // only on request (pace_ps_per_step = -2): on the configurations measured so far the search costs
    // seventy products and has found at most 1.5 %
    const bool wanted = h_opt && h_opt->pace_ps_per_step == -2 && h_opt->barriers != 1 && h_opt->sync_slabs >= 0;
    if (wanted && spmm_desc_get(d_ws, &desc) && desc.mode == 1 && (desc.groups == 2 || desc.groups == 4) &&
        best_ms > 0.f) {
      sagnn_spmm_options o = options_of(best);
      if (o.sync_slabs == 0) o.sync_slabs = 16;
      int rc = spmm_csr_prepare_opt(d_rowptr, d_colidx, d_val, m, k, nnz, f, d_ws, ws_bytes, &o, stream);
      if (rc != SAGNN_OK) { cleanup(); return rc; }
      int32_t best_pace = 0;
      if (spmm_desc_get(d_ws, &desc) && desc.mode == 1 && desc.n_intervals > 1 && desc.mean_steps > 0.f) {
        int dev = 0, cus = 256;
        if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        const int32_t fw = desc.max_slab == 128 && f > 128 ? 128 : (f >= 256 ? 256 : (f >= 128 ? 128 : f));
        const int64_t resident = (int64_t)cus * lds_resident_workgroups((size_t)4 * desc.slots * fw * 4) * 4;
        const double gens = (double)ceil_div(desc.n_waves, resident > 0 ? resident : 1);
        const double ps_hi = (double)best_ms * 1e9 / (gens * (double)desc.mean_steps);
        float paced_best = 0.f, prev = 0.f;
        for (int step = 0; step < 14; ++step) {
          desc.pace_ps_per_step = (int32_t)(ps_hi * (0.96 - 0.04 * step));
          spmm_desc_put(d_ws, desc);
          float ms_min = 0.f;
          for (int rep = 0; rep < 5; ++rep) {
            hipError_t e = hipEventRecord(e0, s);
            if (e != hipSuccess) { set_hip_error(e); cleanup(); return SAGNN_EHIP; }
            rc = launch_spmm(d_rowptr, d_colidx, d_val, m, k, nnz, d_B, ldb, f, d_C, ldc, 0, d_ws, ws_bytes, s);
            if (rc != SAGNN_OK) { cleanup(); return rc; }
            float ms = 0.f;
            e = hipEventRecord(e1, s);
            if (e == hipSuccess) e = hipEventSynchronize(e1);
            if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
            if (e != hipSuccess) { set_hip_error(e); cleanup(); return SAGNN_EHIP; }
            if (rep == 1 || (rep > 1 && ms < ms_min)) ms_min = ms;
          }
          if (paced_best == 0.f || ms_min < paced_best) { paced_best = ms_min; best_pace = desc.pace_ps_per_step; }
          if (prev > 0.f && ms_min > 1.08f * prev) break;    // fell off the schedule: slower again
          prev = ms_min;
        }
        if (paced_best > 0.f && paced_best < 0.985f * best_ms) {
          best_ms = paced_best;
          // one step above the fastest value: a margin against run-to-run variation of the point
          // where the wavefronts stop keeping up
          desc.pace_ps_per_step = best_pace + (int32_t)(ps_hi * 0.02);
          spmm_desc_put(d_ws, desc);
        } else {
          best_pace = 0;
        }
      }
      if (best_pace == 0) {   // restore the layout without intervals
        const sagnn_spmm_options o2 = options_of(best);
        rc = spmm_csr_prepare_opt(d_rowptr, d_colidx, d_val, m, k, nnz, f, d_ws, ws_bytes, &o2, stream);
        if (rc != SAGNN_OK) { cleanup(); return rc; }
      }
    }
  }
  cleanup();
  if (h_choice) {
    h_choice[0] = cand[best].piece;
    h_choice[1] = cand[best].min_long;
    h_choice[2] = (int32_t)(best_ms * 1000.f);
    h_choice[3] = best;
  }
  return SAGNN_OK;
}

SAGNN_EXPORT int spmm_csr_schedule_info(const void* d_ws, int64_t* h_info) {
  using namespace sagnn;
  if (!d_ws || !h_info) return SAGNN_EINVAL;
  SpmmHostDesc d{};
  if (!spmm_desc_get(d_ws, &d)) return SAGNN_EINVAL;
  h_info[0] = d.mode;
  h_info[1] = d.n_waves;
  h_info[2] = d.nnz - (d.mode == 1 ? d.c_nnz : d.nnz);   // entries in the slab-sweep streams
  h_info[3] = d.c_rows;
  h_info[4] = d.c_nnz;
  h_info[5] = d.c_nchunks;
  h_info[6] = d.n_multi_rows;
  h_info[7] = d.has_empty_rows;
  h_info[8] = d.mode == 1 ? d.n_intervals : 0;
  h_info[9] = d.mode == 1 ? d.sync_slabs : 0;
  // byte offset, inside the workspace, of the 32-bit flag the sweep kernels set when a barrier
  // wait ran into its time limit during the most recent product (0 = all barriers were met)
  h_info[10] = (int64_t)(spmm_ws_layout(d.m, d.nnz, d.f).barrier + sizeof(uint32_t) * kSweepBarrierSlots);
  h_info[11] = d.groups;
  h_info[12] = d.mode == 1 ? d.pace_ps_per_step : 0;
  h_info[13] = d.mode == 1 ? d.barriers : 0;
  h_info[14] = d.mode == 1 ? d.slots : 0;
  h_info[15] = d.mode == 1 ? (int64_t)d.max_steps : 0;
  return SAGNN_OK;
}

SAGNN_EXPORT int spmm_csr_tallskinny(const int32_t* d_rowptr, const int32_t* d_colidx,
                                     const float* d_val, int64_t m, int64_t k, int64_t nnz,
                                     const float* d_B, int64_t ldb, int32_t f, float* d_C,
                                     int64_t ldc, int32_t accumulate, void* d_ws, size_t ws_bytes,
                                     void* stream) {
  return sagnn::launch_spmm(d_rowptr, d_colidx, d_val, m, k, nnz, d_B, ldb, f, d_C, ldc,
                            accumulate, d_ws, ws_bytes, (hipStream_t)stream);
}
