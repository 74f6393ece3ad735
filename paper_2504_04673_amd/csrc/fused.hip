// One GCN layer forward in one kernel:  H' = sigma((A H) W)  without the m x f_in intermediate
// T = A H ever reaching HBM (Alg. 1: the statement "Z <- Z + SpMM(..)" followed by
// "H <- GEMM(Z, W)" and the activation; Sec. 2.1 forward equations).
//
// Schedule: row ranges.  A persistent workgroup keeps W in LDS (fp32 [k][n], or bfloat16 packed
// [k/8][n][8]) and walks tiles of RT x 32 consecutive rows of A:
//   phase 1  every wavefront computes whole rows of T for the tile: the row's column ids and
//            values are wavefront-uniform (scalar loads), the 64 lanes split the f_in columns of
//            a row of H, 8 gathers are in flight per wavefront; sums run in blocks of 128
//            entries that are then added up (bounds the length of any serial fp32 sum).  A row
//            with more than kCoopRow entries is shared by all wavefronts of the workgroup
//            (interleaved batches, per-wavefront partial rows in LDS, summed in a fixed order).
//            The row goes to the tile in LDS (fp32, or already rounded to bfloat16 for the
//            bfloat16 product) and, if the caller wants T, to HBM as well.
//   phase 2  wavefront (rt, ct) multiplies the 32 rows of row tile rt by the 32 columns ct of W
//            on the matrix cores (v_mfma_f32_32x32x2_f32 / v_mfma_f32_32x32x16_bf16), applies
//            the activation and stores Z and/or sigma(Z).
// Rows complete inside a workgroup, which is what lets the tile stay on the chip; the price is
// that work is balanced per tile of rows, not per entry.  It suits matrices whose rows are of
// similar length (a partitioned graph's blocks); on power-law matrices the two-kernel path with
// the slab-sweep product is faster and remains the default whenever the caller passes d_T.
#include "common.h"
#include "rowload.h"

namespace sagnn {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kCoopRow = 512;    // rows longer than this are shared by the wavefronts of the workgroup
constexpr int kRunBlock = 128;   // entries per first-level sum
constexpr int kCoopWaves = 8;    // wavefronts that share a long row (one partial row in LDS each)

struct FusedArgs {
  const int32_t* rowptr; const int32_t* colidx; const float* val;
  int64_t m, nnz;
  const float* H; int64_t ldh;
  uint32_t kmax, b_bytes, row_bytes;
  const float* W;
  int32_t f_in, f_out, act;
  float* T; float* Z; float* Hout;
  int32_t rt;          // row tiles (of 32 rows) per workgroup pass
  int32_t nct;         // 32-column tiles of the output
  int32_t ldt;         // elements between two rows of the LDS tile
};

// sum over entries [b, e) taken with stride `stride` batches starting at batch `first`:
// returns this lane's FPL columns of  sum val * H[col, :]
template <int FPL, bool BUF, int U>
__device__ __forceinline__ typename Vec<FPL>::T row_sum(const FusedArgs& g, const int32_t* __restrict__ colidx,
                                                        const float* __restrict__ val,
                                                        const float* __restrict__ H, __amdgpu_buffer_rsrc_t rs,
                                                        int32_t b, int32_t e, int first, int stride,
                                                        uint32_t loff) {
  using vec = typename Vec<FPL>::T;
  vec acc = 0.f, tot = 0.f;
  int since = 0;
  for (int32_t p = b + first * U; p < e; p += stride * U) {
    uint32_t c[U];
    float v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int32_t q = p + u < e ? p + u : e - 1;      // clamped: never reads past the row
      const uint32_t cc = (uint32_t)colidx[q];
      c[u] = cc > g.kmax ? g.kmax : cc;
      v[u] = p + u < e ? val[q] : 0.f;
    }
    vec h[U];
#pragma unroll
    for (int u = 0; u < U; ++u) h[u] = load_row<FPL, BUF>(rs, H, c[u], loff, g.row_bytes, g.ldh);
#pragma unroll
    for (int u = 0; u < U; ++u) asm volatile("" : "+v"(h[u]));
#pragma unroll
    for (int u = 0; u < U; ++u) acc += v[u] * h[u];
    since += U;
    if (since >= kRunBlock) {
      tot += acc;
      acc = 0.f;
      since = 0;
    }
  }
  return tot + acc;
}

// U: gathers a wavefront keeps in flight (16 where the LDS only leaves room for one row tile per pass)
template <int FPL, bool BF16, bool BUF, int U>
__global__ __launch_bounds__(1024) void gcn_fused_kernel(
    // the read-only arrays as separate __restrict__ parameters: that is what lets the compiler
    // fetch the wavefront-uniform row pointers, column ids and values with scalar loads
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx, const float* __restrict__ val,
    const float* __restrict__ H, const float* __restrict__ W, const FusedArgs g) {
  using vec = typename Vec<FPL>::T;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, nthreads = blockDim.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nwaves = nthreads >> 6;
  const int NB = g.nct * 32;                  // padded output width
  const int kdim = g.f_in;                    // 64 * FPL
  // LDS: W slab | tile [rt*32][ldt] | partial rows of a shared long row [<= 8][f_in] | list
  const size_t w_bytes = (size_t)kdim * NB * (BF16 ? 2 : 4);
  char* tile_raw = smem + w_bytes;
  const size_t tile_bytes = (size_t)g.rt * 32 * g.ldt * (BF16 ? 2 : 4);
  float* coop = reinterpret_cast<float*>(tile_raw + tile_bytes);
  const int ncoop = nwaves < kCoopWaves ? nwaves : kCoopWaves;
  int32_t* longlist = reinterpret_cast<int32_t*>(coop + (size_t)ncoop * kdim);   // [0] = count, then local rows

  for (int idx = tid; idx < kdim * NB; idx += nthreads) {
    const int k = idx / NB, n = idx - k * NB;
    const float w = n < g.f_out ? W[(int64_t)k * g.f_out + n] : 0.f;
    if (BF16)
      reinterpret_cast<__bf16*>(smem)[((k >> 3) * NB + n) * 8 + (k & 7)] = (__bf16)w;
    else
      reinterpret_cast<float*>(smem)[k * NB + n] = w;
  }
  const __amdgpu_buffer_rsrc_t rs = make_rsrc(H, g.b_bytes);
  const uint32_t loff = (uint32_t)lane * (FPL * 4);
  const int rows_per_pass = g.rt * 32;
  const int64_t npasses = (g.m + rows_per_pass - 1) / rows_per_pass;

  auto store_tile_row = [&](int lr, vec t) {
    if (BF16) {
      __bf16* p = reinterpret_cast<__bf16*>(tile_raw) + (size_t)lr * g.ldt + lane * FPL;
      if constexpr (FPL == 1) p[0] = (__bf16)t;
      else
#pragma unroll
        for (int i = 0; i < FPL; ++i) p[i] = (__bf16)t[i];
    } else {
      *reinterpret_cast<vec*>(reinterpret_cast<float*>(tile_raw) + (size_t)lr * g.ldt + lane * FPL) = t;
    }
  };

  for (int64_t pass = blockIdx.x; pass < npasses; pass += gridDim.x) {
    const int64_t row0 = pass * rows_per_pass;
    if (tid == 0) {
      longlist[0] = 0;
      longlist[rows_per_pass + 2] = 0;   // next local row to hand out
    }
    __syncthreads();                 // W staged (first pass); previous pass's tile consumed
    // ---- phase 1: T rows of this pass.  A wavefront takes the next row when it is done with its
    // last one (rows differ in length by orders of magnitude on power-law graphs; every row is
    // still summed by one wavefront in a fixed order, so the result does not depend on who took it)
    for (;;) {
      int lr = 0;
      if (lane == 0) lr = atomicAdd(&longlist[rows_per_pass + 2], 1);
      lr = __builtin_amdgcn_readfirstlane(lr);
      if (lr >= rows_per_pass) break;
      const int64_t row = row0 + lr;
      vec t = 0.f;
      bool is_long = false;
      if (row < g.m) {
        int32_t b = rowptr[row], e = rowptr[row + 1];
        b = b < 0 ? 0 : b;
        e = e > g.nnz ? (int32_t)g.nnz : e;
        if (e - b > kCoopRow) {
          is_long = true;
          if (lane == 0) {
            const int slot = atomicAdd(&longlist[0], 1);
            longlist[1 + slot] = lr;
          }
        } else if (e > b) {
          t = row_sum<FPL, BUF, U>(g, colidx, val, H, rs, b, e, 0, 1, loff);
        }
        if (!is_long && g.T) *reinterpret_cast<vec*>(reinterpret_cast<char*>(g.T + row * g.f_in) + loff) = t;
      }
      if (!is_long) store_tile_row(lr, t);
    }
    __syncthreads();
    // rows shared by the whole workgroup, in ascending order of their local index (the list was
    // filled in any order: every wavefront scans for the next smallest, a fixed order)
    const int n_long = longlist[0];
    for (int done = 0, last = -1; done < n_long; ++done) {
      int lr = 0x7FFFFFFF;
      for (int i = 0; i < n_long; ++i) {
        const int x = longlist[1 + i];
        if (x > last && x < lr) lr = x;
      }
      last = lr;
      const int64_t row = row0 + lr;
      int32_t b = rowptr[row], e = rowptr[row + 1];
      b = b < 0 ? 0 : b;
      e = e > g.nnz ? (int32_t)g.nnz : e;
      if (wave < ncoop) {
        const vec part = row_sum<FPL, BUF, U>(g, colidx, val, H, rs, b, e, wave, ncoop, loff);
        *reinterpret_cast<vec*>(coop + (size_t)wave * kdim + lane * FPL) = part;
      }
      __syncthreads();
      if (wave == 0) {
        vec t = 0.f;
        for (int w2 = 0; w2 < ncoop; ++w2) t += *reinterpret_cast<const vec*>(coop + (size_t)w2 * kdim + lane * FPL);
        if (g.T) *reinterpret_cast<vec*>(reinterpret_cast<char*>(g.T + row * g.f_in) + loff) = t;
        store_tile_row(lr, t);
      }
      __syncthreads();
    }
    // ---- phase 2: wavefront (rt, ct) -> one 32 x 32 tile of the output
    {
      const int r = lane & 31, h = lane >> 5;
      for (int tix = wave; tix < g.rt * g.nct; tix += nwaves) {
        const int rtile = tix / g.nct, ct = tix - rtile * g.nct;
        floatx16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
        if (BF16) {
          const bf16x8* __restrict__ Ws = reinterpret_cast<const bf16x8*>(smem);
          const __bf16* trow = reinterpret_cast<const __bf16*>(tile_raw) + (size_t)(rtile * 32 + r) * g.ldt;
          for (int j = 0; j < kdim / 16; ++j) {
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(trow + 16 * j + 8 * h);
            const bf16x8 bb = Ws[(2 * j + h) * NB + ct * 32 + r];
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bb, acc, 0, 0, 0);
          }
        } else {
          const float* __restrict__ Ws = reinterpret_cast<const float*>(smem);
          const float* trow = reinterpret_cast<const float*>(tile_raw) + (size_t)(rtile * 32 + r) * g.ldt;
          for (int j = 0; j < kdim / 8; ++j) {
            const float4 x = *reinterpret_cast<const float4*>(trow + 8 * j + 4 * h);
            const float xs[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
              acc = __builtin_amdgcn_mfma_f32_32x32x2f32(xs[i], Ws[(8 * j + 4 * h + i) * NB + ct * 32 + r], acc, 0, 0, 0);
          }
        }
        const int col = ct * 32 + r;
        if (col < g.f_out) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int64_t ro = row0 + rtile * 32 + (v >> 2) * 8 + h * 4 + (v & 3);
            if (ro >= g.m) continue;
            const float z = acc[v];
            if (g.Z) g.Z[ro * g.f_out + col] = z;
            if (g.Hout) g.Hout[ro * g.f_out + col] = (g.act == SAGNN_ACT_RELU) ? (z > 0.f ? z : 0.f) : z;
          }
        }
      }
    }
  }
}

}  // namespace

namespace {
// row tiles per pass, wavefronts and LDS bytes of a launch; false if W plus one tile do not fit
bool fused_plan(int32_t f_in, int32_t f_out, int32_t prec, int* rt_out, int* waves_out, size_t* lds_out) {
  if (!(f_in == 64 || f_in == 128 || f_in == 256)) return false;
  if (f_out <= 0 || (f_out & 3) || f_out > 256) return false;
  if (prec != SAGNN_GEMM_FP32 && prec != SAGNN_GEMM_BF16) return false;
  const bool bf16 = prec == SAGNN_GEMM_BF16;
  const int nct = (f_out + 31) / 32;
  const int ldt = f_in + (bf16 ? 8 : 4);
  const size_t esz = bf16 ? 2 : 4;
  const size_t w_bytes = (size_t)f_in * nct * 32 * esz;
  // Row tiles per pass: as many as the LDS holds beside W (at most 4).  Wavefronts: 16 whenever
  // they fit (phase 1 is a latency-bound gather: the more rows in flight per CU the better; in
  // phase 2 the wavefronts beyond the number of output tiles of a pass simply have no tile).
  auto lds_for = [&](int r) {
    return w_bytes + (size_t)r * 32 * ldt * esz + (size_t)kCoopWaves * f_in * 4 + 4 * (size_t)(r * 32 + 4);
  };
  int rt = 4;
  while (rt > 1 && lds_for(rt) > 156u * 1024u) --rt;
  if (lds_for(rt) > 156u * 1024u) return false;
  const int waves = 16;
  *rt_out = rt;
  *waves_out = waves;
  *lds_out = lds_for(rt);
  return true;
}
}  // namespace

bool fused_layer_supported(int32_t f_in, int32_t f_out, int32_t prec) {
  int rt = 0, waves = 0;
  size_t lds = 0;
  return fused_plan(f_in, f_out, prec, &rt, &waves, &lds);
}

int launch_fused_layer(const int32_t* rowptr, const int32_t* colidx, const float* val, int64_t m,
                       int64_t k, int64_t nnz, const float* H, int64_t ldh, int32_t f_in,
                       const float* W, int32_t f_out, int32_t act, int32_t prec, float* T, float* Z,
                       float* Hout, hipStream_t s) {
  if (m < 0 || k < 0 || nnz < 0 || m > 0x7FFFFFFFll || k > 0x7FFFFFFFll || nnz > 0x7FFFFFFFll)
    return SAGNN_EINVAL;
  if (prec != SAGNN_GEMM_FP32 && prec != SAGNN_GEMM_BF16) return SAGNN_EINVAL;
  if (act != SAGNN_ACT_IDENTITY && act != SAGNN_ACT_RELU) return SAGNN_EINVAL;
  if (!fused_layer_supported(f_in, f_out, prec)) return SAGNN_EINVAL;
  if (ldh < f_in || (ldh & 3) || !W || (!Z && !Hout)) return SAGNN_EINVAL;
  if (m == 0) return SAGNN_OK;
  if (!rowptr) return SAGNN_EINVAL;
  if (nnz > 0 && (!colidx || !val || !H || !aligned16(H) || k == 0)) return SAGNN_EINVAL;
  const bool bf16 = prec == SAGNN_GEMM_BF16;
  FusedArgs g{};
  g.rowptr = rowptr; g.colidx = colidx; g.val = val; g.m = m; g.nnz = nnz;
  g.H = H; g.ldh = ldh; g.kmax = k > 0 ? (uint32_t)(k - 1) : 0u;
  g.row_bytes = (uint32_t)(ldh * 4);
  const bool buf = buffer_addressable(g.kmax, ldh, f_in, &g.b_bytes);
  g.W = W; g.f_in = f_in; g.f_out = f_out; g.act = act; g.T = T; g.Z = Z; g.Hout = Hout;
  g.nct = (f_out + 31) / 32;
  g.ldt = f_in + (bf16 ? 8 : 4);       // row stride that spreads the rows of a tile over the LDS banks
  int rt = 0, waves = 0;
  size_t lds = 0;
  if (!fused_plan(f_in, f_out, prec, &rt, &waves, &lds)) return SAGNN_EINVAL;
  g.rt = rt;
  const int64_t npasses = ceil_div(m, (int64_t)rt * 32);
  const int per_cu = lds_resident_workgroups(lds) < 1 ? 1 : lds_resident_workgroups(lds);
  int64_t blocks = 256ll * (per_cu > 2 ? 2 : per_cu);
  if (blocks > npasses) blocks = npasses;
  auto go = [&](auto kern) -> int {
    SAGNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(waves * 64), lds, s, rowptr, colidx, val, H, W, g);
    SAGNN_LAUNCH_CHECK();
    return SAGNN_OK;
  };
#define SAGNN_FUSED_U(FPL_, U_)                                                                          \
  (bf16 ? (buf ? go(gcn_fused_kernel<FPL_, true, true, U_>) : go(gcn_fused_kernel<FPL_, true, false, U_>)) \
        : (buf ? go(gcn_fused_kernel<FPL_, false, true, U_>) : go(gcn_fused_kernel<FPL_, false, false, U_>)))
#define SAGNN_FUSED(FPL_) (rt == 1 ? SAGNN_FUSED_U(FPL_, 16) : SAGNN_FUSED_U(FPL_, 8))
  if (f_in == 64) return SAGNN_FUSED(1);
  if (f_in == 128) return SAGNN_FUSED(2);
  return SAGNN_FUSED(4);
#undef SAGNN_FUSED_U
#undef SAGNN_FUSED
}

}  // namespace sagnn
