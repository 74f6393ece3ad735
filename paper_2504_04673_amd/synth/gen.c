/*
 * Seeded synthetic-workload generators (host, plain C + OpenMP).
 *
 * This file only *draws inputs*: random dense matrices, random edge lists and the
 * values of the normalised adjacency matrix.  It holds none of the arithmetic of the
 * method under test (needed-row extraction, row packing, SpMM, GEMM); both the CPU
 * oracle and the GPU library consume the arrays produced here.
 *
 * Every random number is a pure function of (seed, stream, index) through a
 * counter-based generator (SplitMix64 finaliser), so results do not depend on the
 * thread count, on chunking, or on any library's RNG.
 *
 * The graphs stand in for the datasets of the paper's Table 3 (same vertex counts and
 * densities, no dataset content).
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

#define SYNTH_API __attribute__((visibility("default")))

static inline uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

/* counter-based draw: 64 random bits for (seed, stream, idx) */
static inline uint64_t ctr64(uint64_t seed, uint64_t stream, uint64_t idx) {
  uint64_t k = mix64(seed * 0xD1342543DE82EF95ull + mix64(stream));
  return mix64(k ^ mix64(idx));
}

/* uniform double in (0,1): 53 random bits, never 0 or 1 */
static inline double u01(uint64_t bits) {
  return ((double)(bits >> 11) + 0.5) * (1.0 / 9007199254740992.0);
}

SYNTH_API uint64_t synth_ctr64(uint64_t seed, uint64_t stream, uint64_t idx) {
  return ctr64(seed, stream, idx);
}

/* out[i] = lo + (hi-lo) * U(start+i), i in [0,count) */
SYNTH_API void synth_uniform_f32(uint64_t seed, uint64_t stream, uint64_t start,
                                 int64_t count, double lo, double hi, float* out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) {
    double u = u01(ctr64(seed, stream, start + (uint64_t)i));
    out[i] = (float)(lo + (hi - lo) * u);
  }
}

/* standard normal for element index e (Box-Muller in double on the pair e/2) */
static inline double normal_at(uint64_t seed, uint64_t stream, uint64_t e) {
  uint64_t p = e >> 1;
  double u1 = u01(ctr64(seed, stream, 2 * p));
  double u2 = u01(ctr64(seed, stream, 2 * p + 1));
  double r = sqrt(-2.0 * log(u1));
  double t = 6.283185307179586476925286766559 * u2;
  return (e & 1) ? r * sin(t) : r * cos(t);
}

/* out[i] = scale * N(0,1) at element index start+i */
SYNTH_API void synth_normal_f32(uint64_t seed, uint64_t stream, uint64_t start,
                                int64_t count, double scale, float* out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i)
    out[i] = (float)(scale * normal_at(seed, stream, start + (uint64_t)i));
}

/* rows of a virtual (huge) row-major N(0,1) matrix of width f: out[j,:] = M[rows[j],:].
 * Element (r,c) has index r*f+c, so a row's values do not depend on which other rows
 * are materialised. */
SYNTH_API void synth_normal_rows_f32(uint64_t seed, uint64_t stream, const int32_t* rows,
                                     int64_t nrows, int32_t f, double scale, float* out) {
#pragma omp parallel for schedule(static)
  for (int64_t j = 0; j < nrows; ++j) {
    uint64_t base = (uint64_t)(uint32_t)rows[j] * (uint64_t)f;
    for (int32_t c = 0; c < f; ++c)
      out[j * (int64_t)f + c] = (float)(scale * normal_at(seed, stream, base + (uint64_t)c));
  }
}

/* uniform vertex pairs (Erdos-Renyi G(n,M) draws).  key = (min<<32)|max, or ~0 for u==v */
SYNTH_API void synth_uniform_pairs(uint64_t seed, uint64_t stream, uint64_t start,
                                   int64_t count, uint32_t n, uint64_t* keys) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) {
    uint64_t h = ctr64(seed, stream, start + (uint64_t)i);
    uint32_t u = (uint32_t)(((h >> 32) * (uint64_t)n) >> 32);
    uint32_t v = (uint32_t)(((h & 0xFFFFFFFFull) * (uint64_t)n) >> 32);
    if (u == v) { keys[i] = ~0ull; continue; }
    uint32_t a = u < v ? u : v, b = u < v ? v : u;
    keys[i] = ((uint64_t)a << 32) | b;
  }
}

/* bijection on [0, 2^scale): cheap multiply / xor-shift rounds keyed by `key` */
static inline uint32_t relabel(uint32_t x, int scale, uint64_t key) {
  const uint32_t mask = (scale >= 32) ? 0xFFFFFFFFu : ((1u << scale) - 1u);
  const uint32_t m1 = (uint32_t)(mix64(key) | 1u), m2 = (uint32_t)(mix64(key + 1) | 1u);
  const uint32_t a1 = (uint32_t)mix64(key + 2), a2 = (uint32_t)mix64(key + 3);
  const int sh = scale / 2 > 0 ? scale / 2 : 1;
  x = (x * m1 + a1) & mask;
  x ^= x >> sh;
  x = (x * m2 + a2) & mask;
  x ^= x >> sh;
  x = (x * m1 + a2) & mask;
  x ^= x >> sh;
  return x & mask;
}

SYNTH_API uint32_t synth_relabel(uint32_t x, int32_t scale, uint64_t key) {
  return relabel(x, scale, key);
}

/* one R-MAT draw: descend `scale` levels, 16 random bits per level (4 levels per hash).
 * thresholds ta < tb < tc partition [0,65536) into quadrants a | b | c | d. */
static inline void rmat_draw(uint64_t seed, uint64_t stream, uint64_t i, int scale,
                             uint32_t ta, uint32_t tb, uint32_t tc, uint32_t* pu, uint32_t* pv) {
  uint32_t u = 0, v = 0;
  const uint64_t words = (uint64_t)((scale + 3) / 4);
  uint64_t h = 0;
  for (int l = 0; l < scale; ++l) {
    if ((l & 3) == 0) h = ctr64(seed, stream, i * words + (uint64_t)(l >> 2));
    uint32_t r = (uint32_t)(h & 0xFFFFu);
    h >>= 16;
    uint32_t bu = (r >= tb), bv = (r >= ta && r < tb) || (r >= tc);
    u = (u << 1) | bu;
    v = (v << 1) | bv;
  }
  *pu = u; *pv = v;
}

/* R-MAT undirected edge draws start..start+count-1 with vertex relabelling.
 * keys[i] = (min<<32)|max of the relabelled endpoints, or ~0 when the draw is rejected
 * (an endpoint >= n, or a self pair). */
SYNTH_API void synth_rmat_pairs(uint64_t seed, uint64_t stream, uint64_t start, int64_t count,
                                int32_t scale, double a, double b, double c, uint32_t n,
                                uint64_t relabel_key, uint64_t* keys) {
  const uint32_t ta = (uint32_t)(a * 65536.0 + 0.5);
  const uint32_t tb = ta + (uint32_t)(b * 65536.0 + 0.5);
  const uint32_t tc = tb + (uint32_t)(c * 65536.0 + 0.5);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) {
    uint32_t u, v;
    rmat_draw(seed, stream, start + (uint64_t)i, scale, ta, tb, tc, &u, &v);
    u = relabel(u, scale, relabel_key);
    v = relabel(v, scale, relabel_key);
    if (u >= n || v >= n || u == v) { keys[i] = ~0ull; continue; }
    uint32_t lo = u < v ? u : v, hi = u < v ? v : u;
    keys[i] = ((uint64_t)lo << 32) | hi;
  }
}

/* Streaming variant for a graph too large to store: the same draws, but
 *  - every accepted draw adds 1 to deg[u] and deg[v] (draw-level degrees of ALL n
 *    vertices; duplicates are not removed here),
 *  - only entries whose row lies in [r0,r1) are kept: directed keys (row<<32)|col are
 *    appended to out (both orientations when both endpoints are in the block).
 * Returns the number of keys written, or -1 if out_cap would be exceeded.
 * The order of out[] depends on the thread schedule; callers sort it. */
SYNTH_API int64_t synth_rmat_rowblock(uint64_t seed, uint64_t stream, uint64_t start, int64_t count,
                                      int32_t scale, double a, double b, double c, uint32_t n,
                                      uint64_t relabel_key, uint32_t r0, uint32_t r1,
                                      int32_t* deg, uint64_t* out, int64_t out_cap) {
  const uint32_t ta = (uint32_t)(a * 65536.0 + 0.5);
  const uint32_t tb = ta + (uint32_t)(b * 65536.0 + 0.5);
  const uint32_t tc = tb + (uint32_t)(c * 65536.0 + 0.5);
  int64_t pos = 0;
  int overflow = 0;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) {
    uint32_t u, v;
    rmat_draw(seed, stream, start + (uint64_t)i, scale, ta, tb, tc, &u, &v);
    u = relabel(u, scale, relabel_key);
    v = relabel(v, scale, relabel_key);
    if (u >= n || v >= n || u == v) continue;
    if (deg) {
#pragma omp atomic
      deg[u] += 1;
#pragma omp atomic
      deg[v] += 1;
    }
    int inu = (u >= r0 && u < r1), inv = (v >= r0 && v < r1);
    int k = inu + inv;
    if (!k) continue;
    int64_t p;
#pragma omp atomic capture
    { p = pos; pos += k; }
    if (p + k > out_cap) { overflow = 1; continue; }
    if (inu) out[p++] = ((uint64_t)u << 32) | v;
    if (inv) out[p] = ((uint64_t)v << 32) | u;
  }
  return overflow ? -1 : pos;
}

/* Stochastic block model by edge-list sampling.  Vertices [0,n) in `ncomm` equal
 * contiguous communities.  Vertex u draws Poisson(mean_in/2) partners inside its own
 * community and Poisson(mean_out/2) partners outside it, each uniformly; after
 * symmetrisation the expected degrees are mean_in and mean_out.  Up to `kmax` partner
 * slots per vertex and kind; keys[(u*2+kind)*kmax + j] = (min<<32)|max or ~0 if unused. */
static inline int poisson_inv(double mean, double u, int kmax) {
  double p = exp(-mean), cdf = p;
  int k = 0;
  while (u > cdf && k < kmax) { ++k; p *= mean / k; cdf += p; }
  return k;
}

SYNTH_API void synth_sbm_pairs(uint64_t seed, uint64_t stream, uint32_t n, uint32_t ncomm,
                               double mean_in, double mean_out, int32_t kmax, uint64_t* keys) {
  const uint32_t csz = n / ncomm;
#pragma omp parallel for schedule(static)
  for (int64_t u = 0; u < (int64_t)n; ++u) {
    uint32_t g = (uint32_t)u / csz;
    if (g >= ncomm) g = ncomm - 1;
    uint32_t c0 = g * csz, c1 = (g == ncomm - 1) ? n : c0 + csz;
    uint32_t insz = c1 - c0, outsz = n - insz;
    for (int kind = 0; kind < 2; ++kind) {
      uint64_t base = ((uint64_t)u * 2 + (uint64_t)kind) * (uint64_t)(kmax + 1);
      double mean = 0.5 * (kind == 0 ? mean_in : mean_out);
      int k = poisson_inv(mean, u01(ctr64(seed, stream, base)), kmax);
      uint64_t* row = keys + ((uint64_t)u * 2 + (uint64_t)kind) * (uint64_t)kmax;
      for (int j = 0; j < kmax; ++j) {
        if (j >= k) { row[j] = ~0ull; continue; }
        uint64_t h = ctr64(seed, stream, base + 1 + (uint64_t)j);
        uint32_t v;
        if (kind == 0) {
          v = c0 + (uint32_t)(((h >> 32) * (uint64_t)insz) >> 32);
        } else {
          if (outsz == 0) { row[j] = ~0ull; continue; }
          uint32_t t = (uint32_t)(((h >> 32) * (uint64_t)outsz) >> 32);
          v = t < c0 ? t : t + insz;
        }
        if (v == (uint32_t)u) { row[j] = ~0ull; continue; }
        uint32_t lo = (uint32_t)u < v ? (uint32_t)u : v, hi = (uint32_t)u < v ? v : (uint32_t)u;
        row[j] = ((uint64_t)lo << 32) | hi;
      }
    }
  }
}

/* Values of the GCN-normalised adjacency matrix D^-1/2 (A+I) D^-1/2 for a row block:
 * val[e] = (float)(1/sqrt(d_row * d_col)), degrees given for rows (by local index + row0)
 * and columns (global) through one array `deg` of length >= n (double arithmetic). */
SYNTH_API void synth_gcn_values(const int32_t* rowptr, const int32_t* colidx, int64_t m,
                                int64_t row0, const int32_t* deg, float* val) {
#pragma omp parallel for schedule(dynamic, 1024)
  for (int64_t r = 0; r < m; ++r) {
    double dr = (double)deg[row0 + r];
    for (int64_t e = rowptr[r]; e < rowptr[r + 1]; ++e)
      val[e] = (float)(1.0 / sqrt(dr * (double)deg[colidx[e]]));
  }
}

/* split sorted directed keys (row<<32|col, rows relative to row0) into CSR arrays */
SYNTH_API void synth_keys_to_csr(const uint64_t* keys, int64_t nnz, int64_t m, uint32_t row0,
                                 int32_t* rowptr, int32_t* colidx) {
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r <= m; ++r) rowptr[r] = 0;
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < nnz; ++e) {
    colidx[e] = (int32_t)(keys[e] & 0xFFFFFFFFull);
    uint32_t r = (uint32_t)(keys[e] >> 32) - row0;
    /* keys are sorted: row r starts where the row id changes */
    if (e == 0 || (uint32_t)(keys[e - 1] >> 32) - row0 != r) rowptr[r] = (int32_t)e + 1; /* mark start+1 */
  }
  /* rows without entries inherit the next start; fill backwards */
  int32_t next = (int32_t)nnz;
  for (int64_t r = m; r >= 0; --r) {
    if (r == m) { rowptr[r] = (int32_t)nnz; continue; }
    if (rowptr[r] == 0) rowptr[r] = next; else { rowptr[r] -= 1; next = rowptr[r]; }
  }
}
