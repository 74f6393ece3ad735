/*
 * CPU ORACLE -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct definitions of what the GPU library computes.  Nothing
 * in the product path may call this file; only the test-suite, the smoke check and the
 * benchmark's cpu_baseline leg do.  It shares no code, header, table or helper with the
 * HIP sources and includes nothing but the C standard library.
 *
 * What is defined here (paper: "Sparsity-Aware Communication for Distributed Graph
 * Neural Network Training", ICPP'24):
 *   - NnzCols(i,q): the set of nonzero column indices of block (i,q) of the locally
 *     stored sparse row block, i.e. the rows of H_q that process P(i) needs (Sec. 4.1,
 *     the paragraph that introduces NnzCols).
 *   - T = [H[NnzCols(i,0)]; ...; H[NnzCols(i,P-1)]]: the packed row buffer (Alg. 1,
 *     first statement; Alg. 2 "H[srows,:]").
 *   - Z = A_local * H (Alg. 1 "Z <- Z + SpMM(..)", Sec. 4.1 block-sum equation).
 *   - H' = sigma(Z W) (Sec. 2.1 forward equations; Alg. 1 "GEMM(Z, W)").
 *   - G' = (A G W^T) .* sigma'(Z'),  Y = H'^T (A G) (Sec. 2.1 backward equations;
 *     Sec. 4.1 paragraphs on the two gradient equations).
 *
 * Floating point: every sum is accumulated in double, in the stored order of the
 * operands, and rounded to float once.  Each routine can also emit the sum of absolute
 * values of the terms, which the tests use as the scale of the rounding-error bound.
 *
 * Readings where the paper is silent (all listed in the design notes of the repo):
 *   - "nonzero column" is structural: a stored entry counts even if its value is 0;
 *   - indices in NnzCols are global column ids, ascending inside a block, blocks in
 *     ascending order, so the concatenation is globally ascending;
 *   - the diagonal block is packed like every other block;
 *   - sigma is ReLU (flag 1) or the identity (flag 0); sigma'(z) = 1 if z > 0 else 0;
 *   - the modified adjacency matrix is whatever CSR values the caller passes.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_API __attribute__((visibility("default")))

/* ------------------------------------------------------------------------------------
 * NnzCols.  For row block rows [0,m) (the CSR given) and column blocks
 * [colblk[q], colblk[q+1]), q = 0..nb-1 with colblk[0] = 0, colblk[nb] = n:
 *   needed   = ascending list of column ids c that appear in at least one stored entry
 *   blk_off  = nb+1 offsets into needed: block q owns needed[blk_off[q] .. blk_off[q+1])
 *   compact  = for every entry e, the position p with needed[p] == colidx[e]
 * Method: one flag per column, one ascending sweep (brute force by definition).
 * Returns N = blk_off[nb], or -1 on allocation failure / -2 on an index outside [0,n).
 */
ORACLE_API int64_t oracle_needed_rows(const int32_t* rowptr, const int32_t* colidx, int64_t m,
                                      int64_t n, const int64_t* colblk, int32_t nb,
                                      int32_t* needed, int64_t* blk_off, int32_t* compact) {
  unsigned char* flag = (unsigned char*)calloc((size_t)(n > 0 ? n : 1), 1);
  int32_t* pos = compact ? (int32_t*)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1)) : NULL;
  if (!flag || (compact && !pos)) { free(flag); free(pos); return -1; }
  const int64_t nnz = m > 0 ? rowptr[m] : 0;
  for (int64_t e = 0; e < nnz; ++e) {
    int64_t c = colidx[e];
    if (c < 0 || c >= n) { free(flag); free(pos); return -2; }
    flag[c] = 1;
  }
  int64_t N = 0;
  for (int32_t q = 0; q < nb; ++q) {
    blk_off[q] = N;
    for (int64_t c = colblk[q]; c < colblk[q + 1]; ++c)
      if (flag[c]) {
        if (pos) pos[c] = (int32_t)N;
        needed[N++] = (int32_t)c;
      }
  }
  blk_off[nb] = N;
  if (compact)
    for (int64_t e = 0; e < nnz; ++e) compact[e] = pos[colidx[e]];
  free(flag);
  free(pos);
  return N;
}

/* ------------------------------------------------------------------------------------
 * Row pack: out[r, 0:f) = H[rows[r], 0:f), r in [0,N).  Row-major, leading dims ldh, ldo.
 */
ORACLE_API void oracle_pack_rows(const float* H, int64_t ldh, int32_t f, const int32_t* rows,
                                 int64_t N, float* out, int64_t ldo) {
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < N; ++r)
    memcpy(out + r * ldo, H + (int64_t)rows[r] * ldh, sizeof(float) * (size_t)f);
}

/* ------------------------------------------------------------------------------------
 * CSR x dense:  C[r,c] (+)= sum_e val[e] * B[colidx[e], c]  over the entries of row r,
 * in stored order, accumulated in double, rounded once.  With accumulate != 0 the old
 * C[r,c] is the first term of the sum.  Cabs (optional, m x f, ld = f) receives
 * sum_e |val[e]|*|B[..]| (+ |old C|).
 */
ORACLE_API void oracle_spmm(const int32_t* rowptr, const int32_t* colidx, const float* val,
                            int64_t m, const float* B, int64_t ldb, int32_t f, float* C,
                            int64_t ldc, int32_t accumulate, double* Cabs) {
#pragma omp parallel
  {
    double* s = (double*)malloc(sizeof(double) * 2 * (size_t)(f > 0 ? f : 1));
    double* a = s + f;
#pragma omp for schedule(dynamic, 64)
    for (int64_t r = 0; r < m; ++r) {
      for (int32_t c = 0; c < f; ++c) {
        s[c] = accumulate ? (double)C[r * ldc + c] : 0.0;
        a[c] = fabs(s[c]);
      }
      for (int64_t e = rowptr[r]; e < rowptr[r + 1]; ++e) {   /* stored order */
        const double v = (double)val[e];
        const float* brow = B + (int64_t)colidx[e] * ldb;
        for (int32_t c = 0; c < f; ++c) {
          double t = v * (double)brow[c];
          s[c] += t;
          a[c] += fabs(t);
        }
      }
      for (int32_t c = 0; c < f; ++c) {
        C[r * ldc + c] = (float)s[c];
        if (Cabs) Cabs[r * (int64_t)f + c] = a[c];
      }
    }
    free(s);
  }
}

/* round-to-nearest-even float -> bfloat16 -> float (bfloat16 = the upper 16 bits of an
 * IEEE-754 binary32; NaN kept quiet) */
static float bf16_round(float x) {
  uint32_t u;
  memcpy(&u, &x, 4);
  if ((u & 0x7F800000u) == 0x7F800000u) {      /* inf / nan */
    if (u & 0x007FFFFFu) u |= 0x00400000u;
    u &= 0xFFFF0000u;
  } else {
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    u &= 0xFFFF0000u;
  }
  float y;
  memcpy(&y, &u, 4);
  return y;
}

ORACLE_API float oracle_bf16_round(float x) { return bf16_round(x); }

/* ------------------------------------------------------------------------------------
 * Dense product  Z = op(X) * op(W), fp64 accumulation over k ascending, one rounding.
 *   transX == 0: X is m x k (ldx);  transX != 0: X is stored k x m (ldx) and used as X^T
 *   transW == 0: W is k x n (ldw);  transW != 0: W is stored n x k (ldw) and used as W^T
 *   bf16 != 0: both operands are first rounded to bfloat16 (RNE)
 *   Xabs (optional, same shape/stride as X, double, ld = its own row length): replaces |X|
 *        in the magnitude sum, so a caller can propagate the scale of an earlier product
 *   Zabs (optional, m x n, ld = n): sum_k |X|*|W|
 */
ORACLE_API void oracle_gemm(const float* X, int64_t ldx, int32_t transX, const float* W,
                            int64_t ldw, int32_t transW, int64_t m, int64_t k, int64_t n,
                            int32_t bf16, float* Z, int64_t ldz, const double* Xabs,
                            double* Zabs) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < m; ++i) {
    for (int64_t j = 0; j < n; ++j) {
      double s = 0.0, a = 0.0;
      for (int64_t p = 0; p < k; ++p) {
        float x = transX ? X[p * ldx + i] : X[i * ldx + p];
        float w = transW ? W[j * ldw + p] : W[p * ldw + j];
        if (bf16) { x = bf16_round(x); w = bf16_round(w); }
        s += (double)x * (double)w;
        if (Zabs) {
          double xa = Xabs ? (transX ? Xabs[p * m + i] : Xabs[i * k + p]) : fabs((double)x);
          a += xa * fabs((double)w);
        }
      }
      Z[i * ldz + j] = (float)s;
      if (Zabs) Zabs[i * n + j] = a;
    }
  }
}

/* ------------------------------------------------------------------------------------
 * One GCN layer forward (Sec. 2.1 forward equations, in the order of Alg. 1):
 *   T = A * H          (m x f_in)
 *   Z = T * W          (m x f_out)
 *   Hout = act(Z)      act: 0 identity, 1 ReLU
 * Tabs/Zabs optional magnitude companions (Zabs is built from Tabs).
 */
ORACLE_API void oracle_gcn_layer_fwd(const int32_t* rowptr, const int32_t* colidx,
                                     const float* val, int64_t m, const float* H, int64_t ldh,
                                     int32_t f_in, const float* W, int32_t f_out, int32_t act,
                                     int32_t bf16, float* T, float* Z, float* Hout,
                                     double* Tabs, double* Zabs) {
  oracle_spmm(rowptr, colidx, val, m, H, ldh, f_in, T, f_in, 0, Tabs);
  oracle_gemm(T, f_in, 0, W, f_out, 0, m, f_in, f_out, bf16, Z, f_out, Tabs, Zabs);
  const int64_t tot = m * (int64_t)f_out;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < tot; ++i) Hout[i] = (act == 1 && !(Z[i] > 0.0f)) ? 0.0f : Z[i];
}

/* ------------------------------------------------------------------------------------
 * One GCN layer backward (Sec. 2.1 backward equations).  For the layer l with forward
 * Z^l = (A H^{l-1}) W^l and incoming gradient G^l = dLoss/dZ^l:
 *   S     = A_bwd * G^l                       (m x f_out)   "A" of the paper's equation;
 *                                               the caller passes the CSR to multiply by
 *   Gprev = (S * W^T) .* [Zprev > 0]           (m x f_in)    gradient w.r.t. Z^{l-1}
 *                                               (mask skipped when Zprev == NULL)
 *   Y     = Hprev^T * S                        (f_in x f_out) gradient w.r.t. W^l
 * Sabs / Gabs / Yabs: optional magnitude companions.
 */
ORACLE_API void oracle_gcn_layer_bwd(const int32_t* rowptr, const int32_t* colidx,
                                     const float* val, int64_t m, const float* G, int32_t f_out,
                                     const float* W, int32_t f_in, const float* Zprev,
                                     const float* Hprev, int32_t bf16, float* S, float* Gprev,
                                     float* Y, double* Sabs, double* Gabs, double* Yabs) {
  oracle_spmm(rowptr, colidx, val, m, G, f_out, f_out, S, f_out, 0, Sabs);
  if (Gprev) {
    /* W is f_in x f_out row-major; S * W^T uses it transposed */
    oracle_gemm(S, f_out, 0, W, f_out, 1, m, f_out, f_in, bf16, Gprev, f_in, Sabs, Gabs);
    if (Zprev) {
      const int64_t tot = m * (int64_t)f_in;
#pragma omp parallel for schedule(static)
      for (int64_t i = 0; i < tot; ++i)
        if (!(Zprev[i] > 0.0f)) Gprev[i] = 0.0f;
    }
  }
  if (Y) {
    /* Y[a,b] = sum_r Hprev[r,a] * S[r,b]: X = Hprev stored m x f_in used transposed */
    oracle_gemm(Hprev, f_in, 1, S, f_out, 0, f_in, m, f_out, bf16, Y, f_out, NULL, Yabs);
  }
}

ORACLE_API int32_t oracle_max_threads(void) {
#ifdef _OPENMP
  extern int omp_get_max_threads(void);
  return omp_get_max_threads();
#else
  return 1;
#endif
}
