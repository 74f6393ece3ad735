// Dense transforms of the GCN layer on the matrix cores (MFMA), gfx950.
//   forward   Z = T W, H' = sigma(Z)                     (Sec. 2.1 forward equations; Alg. 1
//                                                          "H <- GEMM(Z, W)")
//   backward  G' = (S W^T) .* sigma'(Z')                  (Sec. 2.1 backward equation for G)
//             Y  = H'^T S                                  (Sec. 4.1, weight-gradient paragraph)
//
// Tall-skinny shapes: m is 10^5..10^7 rows, the feature widths are <= 256, so W fits in LDS
// and every kernel streams the tall operand from HBM exactly once.
//
// gemm_nn_kernel (Z = X op(W)): a workgroup stages its slab of W in LDS once and then walks
// row tiles persistently; each wavefront owns a 32-row tile and keeps NT 32x32 accumulator
// tiles in registers.  The A operand of the MFMA is read straight from global memory in
// operand layout: the k order inside an MFMA does not matter as long as both operands agree,
// so lane (row r, half h) takes the 16 (fp32) or 32 (bf16) contiguous bytes
// X[r][8j+4h..] / X[r][16j+8h..] and the matching rows of W are picked from LDS.
//   fp32: v_mfma_f32_32x32x2_f32;  bf16: operands rounded RNE, v_mfma_f32_32x32x16_bf16.
//   fp32 operands as three bfloat16 terms: the same bfloat16 instruction six times per product, W kept in
//   LDS as three packed planes, X split in registers (the accuracy of the fp32 instruction at 6/16 of its cost).
// The epilogue applies the optional mask and activation and stores from the accumulator
// layout (row = 8*(v/4) + 4*(lane/32) + v%4, col = lane%32 of each 32x32 tile).
//
// gemm_tn_kernel (Y = X^T S): the reduction runs over the m rows.  Each workgroup takes a
// contiguous slab of rows, stages 32 rows of X and S at a time in LDS transposed (k
// contiguous per column, so an operand is one LDS read), accumulates a full f_in x f_out
// partial in registers (8 wavefronts x 2x4 tiles) and writes it to scratch; a second kernel
// sums the partials in a fixed order (reproducible, no atomics).
#include <type_traits>

#include "common.h"

namespace sagnn {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct GemmArgs {
  const float* X; int64_t ldx;
  const float* W; int64_t ldw; int32_t transW;
  int64_t m; int32_t kdim, nout;
  int32_t act;
  const float* mask; int64_t ldmask;
  float* Z; int64_t ldz;
  float* A; int64_t lda;
  int32_t n0;  // first output column of this launch's slab
};

// Split mode: a finite fp32 number x is the exact sum of three bfloat16 numbers: t1 = x rounded to
// nearest, t2 = (x - t1) rounded, t3 = x - t1 - t2, which needs no rounding (8 + 8 + 8 significant
// bits); both subtractions are exact, |t2| <= 2^-8 |x| and |t3| <= 2^-16 |x|.
__device__ __forceinline__ void split3(float x, __bf16& t1, __bf16& t2, __bf16& t3) {
  t1 = (__bf16)x;
  const float r = x - (float)t1;
  t2 = (__bf16)r;
  t3 = (__bf16)(r - (float)t2);
}

// ------------------------------------------------------------------------------------------
// KPAD: kdim is not a multiple of 32, loads of X are guarded against the real k extent.
// NG > 0: the k loop has exactly NG groups of 32 and is fully unrolled.  In straight-line code the
// compiler counts outstanding loads exactly; around a loop back-edge it waits for ALL of them,
// which would make the prefetch of the next group useless.
template <int NT, int PREC, int WAVES, bool KPAD, int NG>
__global__ __launch_bounds__(WAVES * 64) void gemm_nn_kernel(const GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int NB = NT * 32;
  constexpr bool BF16 = PREC == SAGNN_GEMM_BF16;
  constexpr bool SPLIT = PREC == SAGNN_GEMM_FP32_BF16X3;
  const int tid = threadIdx.x;
  const int kreal = g.kdim;                  // any multiple of 4
  const int kdim = (kreal + 31) & ~31;       // the k loop runs over the zero-padded extent

  // stage the W slab: fp32 as Ws[k][n]; bf16 packed as Ws[k/8][n][k%8] (split mode: three such
  // planes, one per term); zero outside W
  for (int idx = tid; idx < kdim * NB; idx += WAVES * 64) {
    const int k = idx / NB, n = idx - k * NB;
    const int col = g.n0 + n;
    float w = 0.f;
    if (col < g.nout && k < kreal)
      w = g.transW ? g.W[(int64_t)col * g.ldw + k] : g.W[(int64_t)k * g.ldw + col];
    if (SPLIT) {
      __bf16* Wp = reinterpret_cast<__bf16*>(smem);
      const int at = ((k >> 3) * NB + n) * 8 + (k & 7);
      split3(w, Wp[at], Wp[kdim * NB + at], Wp[2 * kdim * NB + at]);
    } else if (BF16) {
      reinterpret_cast<__bf16*>(smem)[((k >> 3) * NB + n) * 8 + (k & 7)] = (__bf16)w;
    } else {
      reinterpret_cast<float*>(smem)[k * NB + n] = w;
    }
  }
  __syncthreads();

  const int lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, h = lane >> 5;
  const int64_t ntiles = (g.m + 31) >> 5;
  for (int64_t t = (int64_t)blockIdx.x * WAVES + wave; t < ntiles; t += (int64_t)gridDim.x * WAVES) {
    int64_t row = t * 32 + r;
    if (row >= g.m) row = g.m - 1;  // clamped read, result discarded at the store
    const float* __restrict__ xrow = g.X + row * g.ldx;
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
    auto ldx4 = [&](int col) {   // X[row][col..col+3], zero beyond the real k extent
      if constexpr (KPAD) return col < kreal ? *reinterpret_cast<const float4*>(xrow + col) : zero4;
      else return *reinterpret_cast<const float4*>(xrow + col);
    };
    floatx16 acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[nt][v] = 0.f;

    // The k loop runs in groups of JB steps; the A-operand loads of the next group are issued
    // before the MFMAs of the current one, so HBM latency hides behind matrix-core work.
    if (SPLIT) {
      const bf16x8* __restrict__ Ws = reinterpret_cast<const bf16x8*>(smem);
      const int plane = (kdim >> 3) * NB;      // bf16x8 elements per term plane
      constexpr int JB = 2;
      const int ngroups = NG > 0 ? NG : kdim / (16 * JB);
      float4 cur[JB][2], nxt[JB][2];
#pragma unroll
      for (int q = 0; q < JB; ++q) {
        cur[q][0] = ldx4(16 * q + 8 * h);
        cur[q][1] = ldx4(16 * q + 8 * h + 4);
      }
#pragma unroll
      for (int gi = 0; gi < (NG > 0 ? NG : ngroups); ++gi) {
        if (gi + 1 < ngroups) {
#pragma unroll
          for (int q = 0; q < JB; ++q) {
            nxt[q][0] = ldx4(16 * ((gi + 1) * JB + q) + 8 * h);
            nxt[q][1] = ldx4(16 * ((gi + 1) * JB + q) + 8 * h + 4);
          }
        }
        if constexpr (NG > 0) __builtin_amdgcn_sched_barrier(0);   // keep the prefetch ahead of this group's MFMAs
#pragma unroll
        for (int q = 0; q < JB; ++q) {
          const int j = gi * JB + q;
          const float xs[8] = {cur[q][0].x, cur[q][0].y, cur[q][0].z, cur[q][0].w,
                               cur[q][1].x, cur[q][1].y, cur[q][1].z, cur[q][1].w};
          bf16x8 a1, a2, a3;
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            __bf16 t1, t2, t3;
            split3(xs[i], t1, t2, t3);
            a1[i] = t1; a2[i] = t2; a3[i] = t3;
          }
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            const int at = (2 * j + h) * NB + nt * 32 + r;
            const bf16x8 b1 = Ws[at], b2 = Ws[plane + at], b3 = Ws[2 * plane + at];
            // the six products down to 2^-16 of the leading one, smallest first
            acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a3, b1, acc[nt], 0, 0, 0);
            acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b3, acc[nt], 0, 0, 0);
            acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, b2, acc[nt], 0, 0, 0);
            acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, b1, acc[nt], 0, 0, 0);
            acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b2, acc[nt], 0, 0, 0);
            acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, acc[nt], 0, 0, 0);
          }
        }
#pragma unroll
        for (int q = 0; q < JB; ++q) {
          cur[q][0] = nxt[q][0];
          cur[q][1] = nxt[q][1];
        }
      }
    } else if (BF16) {
      const bf16x8* __restrict__ Ws = reinterpret_cast<const bf16x8*>(smem);
      constexpr int JB = 2;
      const int ngroups = NG > 0 ? NG : kdim / (16 * JB);
      float4 cur[JB][2], nxt[JB][2];
#pragma unroll
      for (int q = 0; q < JB; ++q) {
        cur[q][0] = ldx4(16 * q + 8 * h);
        cur[q][1] = ldx4(16 * q + 8 * h + 4);
      }
#pragma unroll
      for (int gi = 0; gi < (NG > 0 ? NG : ngroups); ++gi) {
        if (gi + 1 < ngroups) {
#pragma unroll
          for (int q = 0; q < JB; ++q) {
            nxt[q][0] = ldx4(16 * ((gi + 1) * JB + q) + 8 * h);
            nxt[q][1] = ldx4(16 * ((gi + 1) * JB + q) + 8 * h + 4);
          }
        }
        if constexpr (NG > 0) __builtin_amdgcn_sched_barrier(0);   // keep the prefetch ahead of this group's MFMAs
#pragma unroll
        for (int q = 0; q < JB; ++q) {
          const int j = gi * JB + q;
          const float4 x0 = cur[q][0], x1 = cur[q][1];
          bf16x8 a;
          a[0] = (__bf16)x0.x; a[1] = (__bf16)x0.y; a[2] = (__bf16)x0.z; a[3] = (__bf16)x0.w;
          a[4] = (__bf16)x1.x; a[5] = (__bf16)x1.y; a[6] = (__bf16)x1.z; a[7] = (__bf16)x1.w;
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            const bf16x8 b = Ws[(2 * j + h) * NB + nt * 32 + r];
            acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[nt], 0, 0, 0);
          }
        }
#pragma unroll
        for (int q = 0; q < JB; ++q) {
          cur[q][0] = nxt[q][0];
          cur[q][1] = nxt[q][1];
        }
      }
    } else {
      const float* __restrict__ Ws = reinterpret_cast<const float*>(smem);
      constexpr int JB = 4;
      const int ngroups = NG > 0 ? NG : kdim / (8 * JB);
      float4 cur[JB], nxt[JB];
#pragma unroll
      for (int q = 0; q < JB; ++q) cur[q] = ldx4(8 * q + 4 * h);
#pragma unroll
      for (int gi = 0; gi < (NG > 0 ? NG : ngroups); ++gi) {
        if (gi + 1 < ngroups) {
#pragma unroll
          for (int q = 0; q < JB; ++q)
            nxt[q] = ldx4(8 * ((gi + 1) * JB + q) + 4 * h);
        }
        if constexpr (NG > 0) __builtin_amdgcn_sched_barrier(0);   // keep the prefetch ahead of this group's MFMAs
#pragma unroll
        for (int q = 0; q < JB; ++q) {
          const int j = gi * JB + q;
          const float xs[4] = {cur[q].x, cur[q].y, cur[q].z, cur[q].w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float* wrow = Ws + (8 * j + 4 * h + i) * NB + r;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
              acc[nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(xs[i], wrow[nt * 32], acc[nt], 0, 0, 0);
          }
        }
#pragma unroll
        for (int q = 0; q < JB; ++q) cur[q] = nxt[q];
      }
    }

    if (t * 32 + 32 <= g.m && g.n0 + NB <= g.nout) {
      // full tile: no bounds checks; one base pointer per output array, rows reached by adding
      // the leading dimension (the 16 values of a lane are rows 8*(v/4) + 4*h + v%4)
      const int64_t row0 = t * 32 + h * 4;
      const int col0 = g.n0 + r;
      const float* mk = g.mask ? g.mask + row0 * g.ldmask + col0 : nullptr;
      float* zp = g.Z ? g.Z + row0 * g.ldz + col0 : nullptr;
      float* ap = g.A ? g.A + row0 * g.lda + col0 : nullptr;
      const bool relu = g.act == SAGNN_ACT_RELU;
      if (mk) {
        // the mask is applied in a pass of its own: between the stores below its loads would each
        // have to wait for the store before them (the arrays may alias as far as the compiler
        // knows), one memory round trip per element
        // and its loads are issued a batch at a time (16 to 32 in flight) ahead of their uses
        constexpr int VB = NT >= 8 ? 2 : 4;
#pragma unroll
        for (int v0 = 0; v0 < 16; v0 += VB) {
          float mv[VB][NT];
#pragma unroll
          for (int dv = 0; dv < VB; ++dv) {
            const int64_t dr = ((v0 + dv) >> 2) * 8 + ((v0 + dv) & 3);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) mv[dv][nt] = mk[dr * g.ldmask + nt * 32];
          }
          __builtin_amdgcn_sched_barrier(0);   // keep the batch of loads together, ahead of the selects
#pragma unroll
          for (int dv = 0; dv < VB; ++dv)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
              if (!(mv[dv][nt] > 0.f)) acc[nt][v0 + dv] = 0.f;
        }
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t dr = (v >> 2) * 8 + (v & 3);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          const float z = acc[nt][v];
          if (zp) zp[dr * g.ldz + nt * 32] = z;
          if (ap) ap[dr * g.lda + nt * 32] = relu ? (z > 0.f ? z : 0.f) : z;
        }
      }
    } else {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const int col = g.n0 + nt * 32 + r;
        if (col >= g.nout) continue;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int64_t ro = t * 32 + (v >> 2) * 8 + h * 4 + (v & 3);
          if (ro >= g.m) continue;
          float z = acc[nt][v];
          if (g.mask && !(g.mask[ro * g.ldmask + col] > 0.f)) z = 0.f;
          if (g.Z) g.Z[ro * g.ldz + col] = z;
          if (g.A) g.A[ro * g.lda + col] = (g.act == SAGNN_ACT_RELU) ? (z > 0.f ? z : 0.f) : z;
        }
      }
    }
  }
}

template <int NT, int PREC, int WAVES>
int launch_nn_waves(const GemmArgs& g, size_t lds, hipStream_t s) {
  void (*kern)(const GemmArgs) = gemm_nn_kernel<NT, PREC, WAVES, false, 0>;
  if (g.kdim & 31) kern = gemm_nn_kernel<NT, PREC, WAVES, true, 0>;
  else if (g.kdim == 128) kern = gemm_nn_kernel<NT, PREC, WAVES, false, 4>;
  else if (g.kdim == 256) kern = gemm_nn_kernel<NT, PREC, WAVES, false, 8>;
  SAGNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  const int64_t ntiles = (g.m + 31) / 32;
  int64_t blocks = ceil_div(ntiles, WAVES);
  const int64_t per_cu = lds > 80 * 1024 ? 1 : (lds > 40 * 1024 ? 2 : 4);
  if (blocks > 256 * per_cu) blocks = 256 * per_cu;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(WAVES * 64), lds, s, g);
  SAGNN_LAUNCH_CHECK();
  return SAGNN_OK;
}

// bytes of LDS the W slab of NT*32 columns takes (split mode: three bfloat16 planes)
inline size_t nn_slab_bytes(int32_t kdim, int nt, int prec) {
  const size_t elems = (size_t)((kdim + 31) & ~31) * nt * 32;
  return prec == SAGNN_GEMM_FP32 ? elems * 4 : (prec == SAGNN_GEMM_BF16 ? elems * 2 : elems * 6);
}

template <int NT, int PREC>
int launch_nn(const GemmArgs& g, hipStream_t s) {
  const size_t lds = nn_slab_bytes(g.kdim, NT, PREC);
  if (lds > 160 * 1024) return SAGNN_EINVAL;
  // fp32: 4 wavefronts per workgroup, two workgroups per CU while the W slab allows it; when the
  // slab is so large that only one workgroup fits a CU, 8 wavefronts keep two per SIMD
  if (PREC != SAGNN_GEMM_FP32 || lds > 80 * 1024) return launch_nn_waves<NT, PREC, 8>(g, lds, s);
  return launch_nn_waves<NT, PREC, 4>(g, lds, s);
}

// ------------------------------------------------------------------------------------------
// Y = X^T S.  KB rows per stage; LDS rows padded to KP elements (16-byte multiple).
constexpr int kTnWaves = 8;
constexpr int kTnThreads = kTnWaves * 64;
constexpr int KB = 32, KP = 40;

struct TnArgs {
  const float* X; int64_t ldx;
  const float* S; int64_t lds_;
  int64_t m; int32_t fi, fo;
  int64_t rows_per_wg;
  float* partial;  // [gridDim.x][fi][fo]
};

// PREC as in gemm_nn_kernel; PREC = 2 keeps three bfloat16 planes (one per term) of both staged operands
template <int PREC>
__global__ __launch_bounds__(kTnThreads) void gemm_tn_kernel(const TnArgs g) {
  constexpr bool BF16 = PREC == SAGNN_GEMM_BF16;
  constexpr bool X3 = PREC == SAGNN_GEMM_FP32_BF16X3;
  using lds_t = typename std::conditional<PREC != SAGNN_GEMM_FP32, __bf16, float>::type;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  lds_t* Xs = reinterpret_cast<lds_t*>(smem);                    // [fi][KP]
  lds_t* Ss = Xs + (size_t)((g.fi + 31) / 32) * 32 * KP;         // [fo][KP], after the padded X part
  const int plane = ((g.fi + 31) / 32 + (g.fo + 31) / 32) * 32 * KP;   // elements per term plane (X3)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i = lane & 31, h = lane >> 5;
  const int wa = wave >> 1, wb = wave & 1;  // wave tile: a-tiles {2wa,2wa+1}, b-tiles {4wb..4wb+3}
  const int TA = (g.fi + 31) / 32, TB = (g.fo + 31) / 32;
  // columns of the last tile that lie beyond fi / fo are never staged: keep them zero
  for (int idx = tid; idx < (TA + TB) * 32 * KP * (X3 ? 3 : 1); idx += kTnThreads) Xs[idx] = (lds_t)0.f;
  __syncthreads();

  const int64_t r_begin = (int64_t)blockIdx.x * g.rows_per_wg;
  int64_t r_end = r_begin + g.rows_per_wg;
  if (r_end > g.m) r_end = g.m;

  floatx16 acc[2][4];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  // staging map: thread -> (column group cg of 4 columns, row pair kp); 64 groups x 8 pairs
  // per pass, two passes cover the KB = 32 rows of a stage
  const int cg = tid & 63, kp = tid >> 6;
  float4 xr[2][2], sr[2][2];
  auto load_stage = [&](int64_t r0) {
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int64_t row = r0 + (kp + 8 * p) * 2 + q;
        const bool ok = row < r_end;
        xr[p][q] = (ok && cg * 4 < g.fi) ? *reinterpret_cast<const float4*>(g.X + row * g.ldx + cg * 4)
                                         : make_float4(0.f, 0.f, 0.f, 0.f);
        sr[p][q] = (ok && cg * 4 < g.fo) ? *reinterpret_cast<const float4*>(g.S + row * g.lds_ + cg * 4)
                                         : make_float4(0.f, 0.f, 0.f, 0.f);
      }
  };
  // Transposing stores: column col = 4 cg + c of the stage goes to LDS row col, k contiguous, so a
  // lane's two rows (k, k + 1) of one column are one 4-byte (bfloat16) or 8-byte (fp32) store.  Row
  // starts are 20 (40) words apart: lanes that store the same c fall on two banks only.  Lane cg
  // therefore takes its four columns in the order c = (j + cg / 2) mod 4, which spreads a store over
  // eight banks.
  auto pick = [](const float (&a)[4], int c) { return c == 0 ? a[0] : (c == 1 ? a[1] : (c == 2 ? a[2] : a[3])); };
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  auto store_stage = [&]() {
    // (rounded-bfloat16 mode: the stage is short and bound by the latency of its loads; the selects of
    // the rotation would only lengthen the path from a load to its store)
    const int rot = BF16 ? 0 : (cg >> 1) & 3;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const int kk = (kp + 8 * p) * 2;
      const float xa[4] = {xr[p][0].x, xr[p][0].y, xr[p][0].z, xr[p][0].w};
      const float xb[4] = {xr[p][1].x, xr[p][1].y, xr[p][1].z, xr[p][1].w};
      const float sa[4] = {sr[p][0].x, sr[p][0].y, sr[p][0].z, sr[p][0].w};
      const float sb[4] = {sr[p][1].x, sr[p][1].y, sr[p][1].z, sr[p][1].w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int c = BF16 ? j : (j + rot) & 3;
        const int col = cg * 4 + c;
        const float x0 = BF16 ? xa[j] : pick(xa, c), x1 = BF16 ? xb[j] : pick(xb, c);
        const float s0 = BF16 ? sa[j] : pick(sa, c), s1 = BF16 ? sb[j] : pick(sb, c);
        if constexpr (X3) {
          __bf16* Xb = reinterpret_cast<__bf16*>(Xs);
          __bf16* Sb = reinterpret_cast<__bf16*>(Ss);
          __bf16 lo[3], hi[3];
          if (col < g.fi) {
            split3(x0, lo[0], lo[1], lo[2]);
            split3(x1, hi[0], hi[1], hi[2]);
#pragma unroll
            for (int q = 0; q < 3; ++q) {
              bf16x2 t;
              t[0] = lo[q]; t[1] = hi[q];
              *reinterpret_cast<bf16x2*>(Xb + q * plane + col * KP + kk) = t;
            }
          }
          if (col < g.fo) {
            split3(s0, lo[0], lo[1], lo[2]);
            split3(s1, hi[0], hi[1], hi[2]);
#pragma unroll
            for (int q = 0; q < 3; ++q) {
              bf16x2 t;
              t[0] = lo[q]; t[1] = hi[q];
              *reinterpret_cast<bf16x2*>(Sb + q * plane + col * KP + kk) = t;
            }
          }
        } else if constexpr (BF16) {
          __bf16* Xb = reinterpret_cast<__bf16*>(Xs);
          __bf16* Sb = reinterpret_cast<__bf16*>(Ss);
          bf16x2 t;
          if (col < g.fi) {
            t[0] = (__bf16)x0; t[1] = (__bf16)x1;
            *reinterpret_cast<bf16x2*>(Xb + col * KP + kk) = t;
          }
          if (col < g.fo) {
            t[0] = (__bf16)s0; t[1] = (__bf16)s1;
            *reinterpret_cast<bf16x2*>(Sb + col * KP + kk) = t;
          }
        } else {
          float* Xf = reinterpret_cast<float*>(Xs);
          float* Sf = reinterpret_cast<float*>(Ss);
          if (col < g.fi) *reinterpret_cast<float2*>(Xf + col * KP + kk) = make_float2(x0, x1);
          if (col < g.fo) *reinterpret_cast<float2*>(Sf + col * KP + kk) = make_float2(s0, s1);
        }
      }
    }
  };

  if (r_begin < r_end) load_stage(r_begin);
  for (int64_t r0 = r_begin; r0 < r_end; r0 += KB) {
    __syncthreads();  // previous stage fully consumed
    store_stage();
    __syncthreads();
    if (r0 + KB < r_end) load_stage(r0 + KB);  // prefetch the next stage into registers
    if constexpr (X3) {
      const __bf16* Xb = reinterpret_cast<const __bf16*>(Xs);
      const __bf16* Sb = reinterpret_cast<const __bf16*>(Ss);
#pragma unroll 1
      for (int ks = 0; ks < KB / 16; ++ks) {
        // (the terms of one operand pair at a time: 128 accumulator registers leave room for little else)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const int tb = 4 * wb + b;
          bf16x8 bv[3];
#pragma unroll
          for (int t = 0; t < 3; ++t)
            bv[t] = *reinterpret_cast<const bf16x8*>(Sb + t * plane + ((tb < TB ? tb : 0) * 32 + i) * KP + ks * 16 + 8 * h);
#pragma unroll
          for (int a = 0; a < 2; ++a) {
            const int ta = 2 * wa + a;
            bf16x8 av[3];
#pragma unroll
            for (int t = 0; t < 3; ++t)
              av[t] = *reinterpret_cast<const bf16x8*>(Xb + t * plane + ((ta < TA ? ta : 0) * 32 + i) * KP + ks * 16 + 8 * h);
            if (ta < TA && tb < TB) {
              // the six products down to 2^-16 of the leading one, smallest first
              acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[2], bv[0], acc[a][b], 0, 0, 0);
              acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[0], bv[2], acc[a][b], 0, 0, 0);
              acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[1], bv[1], acc[a][b], 0, 0, 0);
              acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[1], bv[0], acc[a][b], 0, 0, 0);
              acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[0], bv[1], acc[a][b], 0, 0, 0);
              acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[0], bv[0], acc[a][b], 0, 0, 0);
            }
          }
        }
      }
    } else if (BF16) {
#pragma unroll
      for (int ks = 0; ks < KB / 16; ++ks) {
        bf16x8 av[2], bv[4];
#pragma unroll
        for (int a = 0; a < 2; ++a) {
          const int ta = 2 * wa + a;
          av[a] = *reinterpret_cast<const bf16x8*>(
              reinterpret_cast<const __bf16*>(Xs) + ((ta < TA ? ta : 0) * 32 + i) * KP + ks * 16 + 8 * h);
        }
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const int tb = 4 * wb + b;
          bv[b] = *reinterpret_cast<const bf16x8*>(
              reinterpret_cast<const __bf16*>(Ss) + ((tb < TB ? tb : 0) * 32 + i) * KP + ks * 16 + 8 * h);
        }
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
          for (int b = 0; b < 4; ++b)
            if (2 * wa + a < TA && 4 * wb + b < TB)
              acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[a], bv[b], acc[a][b], 0, 0, 0);
      }
    } else {
#pragma unroll 4
      for (int ks = 0; ks < KB / 2; ++ks) {
        float av[2], bv[4];
#pragma unroll
        for (int a = 0; a < 2; ++a) {
          const int ta = 2 * wa + a;
          av[a] = reinterpret_cast<const float*>(Xs)[((ta < TA ? ta : 0) * 32 + i) * KP + ks * 2 + h];
        }
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const int tb = 4 * wb + b;
          bv[b] = reinterpret_cast<const float*>(Ss)[((tb < TB ? tb : 0) * 32 + i) * KP + ks * 2 + h];
        }
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
          for (int b = 0; b < 4; ++b)
            if (2 * wa + a < TA && 4 * wb + b < TB)
              acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[a], bv[b], acc[a][b], 0, 0, 0);
      }
    }
  }

  float* __restrict__ P = g.partial + (int64_t)blockIdx.x * g.fi * g.fo;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const int ta = 2 * wa + a, tb = 4 * wb + b;
      if (ta >= TA || tb >= TB) continue;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int ro = ta * 32 + (v >> 2) * 8 + h * 4 + (v & 3);
        if (ro < g.fi && tb * 32 + i < g.fo) P[(int64_t)ro * g.fo + tb * 32 + i] = acc[a][b][v];
      }
    }
}

__global__ __launch_bounds__(256) void tn_reduce_kernel(const float* __restrict__ partial,
                                                        int32_t nparts, int64_t elems,
                                                        float* __restrict__ Y) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= elems) return;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  int p = 0;
  for (; p + 4 <= nparts; p += 4) {
    s0 += partial[(int64_t)(p + 0) * elems + idx];
    s1 += partial[(int64_t)(p + 1) * elems + idx];
    s2 += partial[(int64_t)(p + 2) * elems + idx];
    s3 += partial[(int64_t)(p + 3) * elems + idx];
  }
  for (; p < nparts; ++p) s0 += partial[(int64_t)p * elems + idx];
  Y[idx] = (s0 + s1) + (s2 + s3);
}

inline int32_t tn_parts(int64_t m) {
  int64_t p = ceil_div(m, 4 * KB);  // at least 4 stages of work per workgroup
  if (p > 256) p = 256;
  if (p < 1) p = 1;
  return (int32_t)p;
}

}  // namespace

size_t gemm_tn_ws_bytes(int64_t m, int32_t fi, int32_t fo) {
  return round_up(sizeof(float) * (size_t)tn_parts(m) * (size_t)fi * (size_t)fo, 256);
}

int launch_gemm_tn(const float* X, int64_t ldx, const float* S, int64_t lds_, int64_t m,
                   int32_t fi, int32_t fo, int32_t prec, float* Y, void* yws, size_t yws_bytes,
                   hipStream_t s) {
  if (m < 0 || fi <= 0 || fo <= 0 || (fi & 3) || (fo & 3) || fi > 256 || fo > 256 ||
      ldx < fi || lds_ < fo || (ldx & 3) || (lds_ & 3))
    return SAGNN_EINVAL;
  if (prec != SAGNN_GEMM_FP32 && prec != SAGNN_GEMM_BF16 && prec != SAGNN_GEMM_FP32_BF16X3) return SAGNN_EINVAL;
  if (!Y || !yws || !aligned16(yws)) return SAGNN_EINVAL;
  if (m > 0 && (!X || !S || !aligned16(X) || !aligned16(S))) return SAGNN_EINVAL;
  if (yws_bytes < gemm_tn_ws_bytes(m, fi, fo)) return SAGNN_ECAPACITY;
  const int32_t parts = tn_parts(m);
  TnArgs g{};
  g.X = X; g.ldx = ldx; g.S = S; g.lds_ = lds_; g.m = m; g.fi = fi; g.fo = fo;
  g.rows_per_wg = ceil_div(ceil_div(m > 0 ? m : 1, parts), KB) * KB;
  g.partial = reinterpret_cast<float*>(yws);
  const size_t lds = (size_t)(((fi + 31) / 32 + (fo + 31) / 32) * 32) * KP *
                     (prec == SAGNN_GEMM_BF16 ? 2 : (prec == SAGNN_GEMM_FP32_BF16X3 ? 6 : 4));
  auto go = [&](auto kern) -> int {
    SAGNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)lds));
    hipLaunchKernelGGL(kern, dim3(parts), dim3(kTnThreads), lds, s, g);
    return SAGNN_OK;
  };
  int rc;
  if (prec == SAGNN_GEMM_BF16) rc = go(gemm_tn_kernel<SAGNN_GEMM_BF16>);
  else if (prec == SAGNN_GEMM_FP32_BF16X3) rc = go(gemm_tn_kernel<SAGNN_GEMM_FP32_BF16X3>);
  else rc = go(gemm_tn_kernel<SAGNN_GEMM_FP32>);
  if (rc != SAGNN_OK) return rc;
  SAGNN_LAUNCH_CHECK();
  const int64_t elems = (int64_t)fi * fo;
  hipLaunchKernelGGL(tn_reduce_kernel, dim3((unsigned)ceil_div(elems, 256)), dim3(256), 0, s,
                     g.partial, parts, elems, Y);
  SAGNN_LAUNCH_CHECK();
  return SAGNN_OK;
}

int launch_gemm(const float* X, int64_t ldx, const float* W, int64_t ldw, int32_t transW,
                int64_t m, int32_t kdim, int32_t nout, int32_t prec, int32_t act,
                const float* mask, int64_t ldmask, float* Z, int64_t ldz, float* A, int64_t lda,
                hipStream_t s) {
  if (m < 0 || kdim <= 0 || nout <= 0 || (kdim & 3) || (nout & 3) || kdim > 256 || nout > 256)
    return SAGNN_EINVAL;
  if (prec != SAGNN_GEMM_FP32 && prec != SAGNN_GEMM_BF16 && prec != SAGNN_GEMM_FP32_BF16X3) return SAGNN_EINVAL;
  if (act != SAGNN_ACT_IDENTITY && act != SAGNN_ACT_RELU) return SAGNN_EINVAL;
  if (transW != 0 && transW != 1) return SAGNN_EINVAL;
  if (ldx < kdim || (ldx & 3) || ldw < (transW ? kdim : nout)) return SAGNN_EINVAL;
  if ((Z && ldz < nout) || (A && lda < nout) || (mask && ldmask < nout)) return SAGNN_EINVAL;
  if (!Z && !A) return SAGNN_EINVAL;
  if (!W) return SAGNN_EINVAL;
  if (m == 0) return SAGNN_OK;
  if (!X || !aligned16(X)) return SAGNN_EINVAL;

  GemmArgs g{};
  g.X = X; g.ldx = ldx; g.W = W; g.ldw = ldw; g.transW = transW; g.m = m; g.kdim = kdim;
  g.nout = nout; g.act = act; g.mask = mask; g.ldmask = ldmask; g.Z = Z; g.ldz = ldz; g.A = A;
  g.lda = lda;
  if (prec == SAGNN_GEMM_BF16) {
    g.n0 = 0;
    const int tiles = (nout + 31) / 32;
    if (tiles <= 1) return launch_nn<1, SAGNN_GEMM_BF16>(g, s);
    if (tiles <= 2) return launch_nn<2, SAGNN_GEMM_BF16>(g, s);
    if (tiles <= 4) return launch_nn<4, SAGNN_GEMM_BF16>(g, s);
    return launch_nn<8, SAGNN_GEMM_BF16>(g, s);
  }
  if (prec == SAGNN_GEMM_FP32_BF16X3) {
    // the widest column slab whose three planes fit the LDS: 128 columns up to k = 128, 64 beyond
    const int32_t slab = nn_slab_bytes(kdim, 4, prec) <= 160 * 1024 ? 128 : 64;
    for (int32_t n0 = 0; n0 < nout; n0 += slab) {
      g.n0 = n0;
      const int tiles = ((nout - n0 < slab ? nout - n0 : slab) + 31) / 32;
      int rc;
      if (tiles <= 1) rc = launch_nn<1, SAGNN_GEMM_FP32_BF16X3>(g, s);
      else if (tiles <= 2) rc = launch_nn<2, SAGNN_GEMM_FP32_BF16X3>(g, s);
      else rc = launch_nn<4, SAGNN_GEMM_FP32_BF16X3>(g, s);
      if (rc != SAGNN_OK) return rc;
    }
    return SAGNN_OK;
  }
  for (int32_t n0 = 0; n0 < nout; n0 += 128) {
    g.n0 = n0;
    const int tiles = ((nout - n0 < 128 ? nout - n0 : 128) + 31) / 32;
    int rc;
    if (tiles <= 1) rc = launch_nn<1, SAGNN_GEMM_FP32>(g, s);
    else if (tiles <= 2) rc = launch_nn<2, SAGNN_GEMM_FP32>(g, s);
    else rc = launch_nn<4, SAGNN_GEMM_FP32>(g, s);
    if (rc != SAGNN_OK) return rc;
  }
  return SAGNN_OK;
}

}  // namespace sagnn

SAGNN_EXPORT int dense_gemm_act(const float* d_X, int64_t ldx, const float* d_W, int64_t ldw,
                                int32_t transW, int64_t m, int32_t kdim, int32_t nout,
                                int32_t prec, int32_t act, const float* d_mask, int64_t ldmask,
                                float* d_Z, int64_t ldz, float* d_act, int64_t ldact,
                                void* stream) {
  return sagnn::launch_gemm(d_X, ldx, d_W, ldw, transW, m, kdim, nout, prec, act, d_mask, ldmask,
                            d_Z, ldz, d_act, ldact, (hipStream_t)stream);
}
