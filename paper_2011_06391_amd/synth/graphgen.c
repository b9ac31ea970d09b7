/*
 * Seeded synthetic workload generators: graphs (Erdos-Renyi, R-MAT, Chung-Lu),
 * CSR assembly and dense feature fills.
 *
 * This file produces INPUTS only.  It contains none of the arithmetic of the
 * fused SDDMM-SpMM method: no VOP/ROP/SOP/MOP/AOP step is computed here.  The
 * GPU library and the CPU oracle both receive the arrays made here; neither
 * includes or links this file for any other purpose.
 *
 * Every random quantity is a pure function of (seed, stream, index) through a
 * counter-based generator, so results do not depend on thread count, on the
 * order in which OpenMP threads run, or on any library's generator.
 *
 * Plain C + OpenMP, built with gcc into libgraphgen.so.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- counter-based generator: two rounds of the splitmix64 finaliser ---- */
static inline uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ULL;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
  return z ^ (z >> 31);
}

static inline uint64_t ctr_u64(uint64_t seed, uint64_t stream, uint64_t idx) {
  return mix64(mix64(seed ^ mix64(stream)) + idx);
}

/* uniform double in [0,1) with 53 random bits */
static inline double ctr_u01(uint64_t seed, uint64_t stream, uint64_t idx) {
  return (double)(ctr_u64(seed, stream, idx) >> 11) * (1.0 / 9007199254740992.0);
}

uint64_t synth_ctr_u64(uint64_t seed, uint64_t stream, uint64_t idx) {
  return ctr_u64(seed, stream, idx);
}

/* ---- dense fills ---------------------------------------------------------- */

/* out[i] = lo + (hi-lo) * k/2^24, k = top 24 bits of the counter draw: every
 * value is exactly representable in fp32 and lies in [lo, hi). */
void synth_fill_uniform(float* out, int64_t count, uint64_t seed, float lo, float hi) {
  const float scale = (hi - lo) * (1.0f / 16777216.0f);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) {
    uint32_t k = (uint32_t)(ctr_u64(seed, 0, (uint64_t)i) >> 40);
    out[i] = lo + scale * (float)k;
  }
}

/* Standard normal by Box-Muller on two counter draws per output. */
void synth_fill_normal(float* out, int64_t count, uint64_t seed) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) {
    double u1 = ctr_u01(seed, 1, (uint64_t)i);
    double u2 = ctr_u01(seed, 2, (uint64_t)i);
    u1 = 1.0 - u1; /* (0,1] so the log is finite */
    out[i] = (float)(sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2));
  }
}

/* Integers drawn uniformly from [lo, hi], stored as floats (for tests whose
 * fp32 sums must be exact in any order). */
void synth_fill_int(float* out, int64_t count, uint64_t seed, int32_t lo, int32_t hi) {
  const uint64_t span = (uint64_t)(hi - lo + 1);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) {
    uint64_t r = ctr_u64(seed, 3, (uint64_t)i) >> 16;
    out[i] = (float)(lo + (int32_t)(r % span));
  }
}

/* ---- vertex relabelling ---------------------------------------------------- */

typedef struct { uint64_t key; int32_t id; } keyed_t;

static int cmp_keyed(const void* a, const void* b) {
  const keyed_t* x = (const keyed_t*)a;
  const keyed_t* y = (const keyed_t*)b;
  if (x->key < y->key) return -1;
  if (x->key > y->key) return 1;
  return (x->id > y->id) - (x->id < y->id);
}

/* perm[old] = new label; a permutation obtained by ranking one counter draw
 * per vertex.  Returns 0, or -1 when out of memory. */
int synth_permutation(int64_t n, uint64_t seed, int32_t* perm) {
  keyed_t* k = (keyed_t*)malloc((size_t)n * sizeof(keyed_t));
  if (!k) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    k[i].key = ctr_u64(seed, 4, (uint64_t)i);
    k[i].id = (int32_t)i;
  }
  qsort(k, (size_t)n, sizeof(keyed_t), cmp_keyed);
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < n; ++r) perm[k[r].id] = (int32_t)r;
  free(k);
  return 0;
}

/* ---- edge-pair generators (each writes npairs (src,dst) pairs) ------------- */

/* R-MAT: at each of `scale` levels one counter draw picks a quadrant with
 * probabilities (a, b, c, 1-a-b-c); quadrant bits build (src, dst).  No noise
 * is added to the probabilities. */
void synth_rmat_pairs(int32_t scale, int64_t npairs, double a, double b, double c,
                      uint64_t seed, int32_t* src, int32_t* dst) {
  const double ab = a + b, abc = a + b + c;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < npairs; ++i) {
    uint32_t u = 0, v = 0;
    for (int32_t level = 0; level < scale; ++level) {
      double r = ctr_u01(seed, 16 + (uint64_t)level, (uint64_t)i);
      uint32_t ub, vb;
      if (r < a) { ub = 0; vb = 0; }
      else if (r < ab) { ub = 0; vb = 1; }
      else if (r < abc) { ub = 1; vb = 0; }
      else { ub = 1; vb = 1; }
      u = (u << 1) | ub;
      v = (v << 1) | vb;
    }
    src[i] = (int32_t)u;
    dst[i] = (int32_t)v;
  }
}

/* Chung-Lu by independent endpoint sampling: both endpoints of each pair are
 * drawn from the density proportional to (x + i0)^(-1/2) on [0, n), floored to
 * a vertex id, by inverting its closed-form CDF. */
void synth_chunglu_pairs(int64_t n, int64_t npairs, double i0, uint64_t seed,
                         int32_t* src, int32_t* dst) {
  const double r0 = sqrt(i0), r1 = sqrt((double)n + i0);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < npairs; ++i) {
    for (int side = 0; side < 2; ++side) {
      double u = ctr_u01(seed, 8 + (uint64_t)side, (uint64_t)i);
      double r = r0 + u * (r1 - r0);
      int64_t id = (int64_t)floor(r * r - i0);
      if (id < 0) id = 0;
      if (id >= n) id = n - 1;
      if (side == 0) src[i] = (int32_t)id; else dst[i] = (int32_t)id;
    }
  }
}

/* Erdos-Renyi G(n, M): the first M distinct unordered non-loop pairs of the
 * counter stream.  Sequential (used for small graphs only).  Returns the
 * number of pairs written (== M unless M exceeds n(n-1)/2), or -1 on
 * allocation failure. */
int64_t synth_er_pairs(int64_t n, int64_t M, uint64_t seed, int32_t* src, int32_t* dst) {
  if (n < 2 || M <= 0) return 0;
  const int64_t max_pairs = n * (n - 1) / 2;
  if (M > max_pairs) M = max_pairs;
  uint64_t cap = 16;
  while (cap < (uint64_t)M * 4) cap <<= 1;
  uint64_t* table = (uint64_t*)malloc(cap * sizeof(uint64_t));
  if (!table) return -1;
  memset(table, 0xFF, cap * sizeof(uint64_t));
  int64_t got = 0;
  for (uint64_t draw = 0; got < M; ++draw) {
    uint64_t a = ctr_u64(seed, 5, draw) % (uint64_t)n;
    uint64_t b = ctr_u64(seed, 6, draw) % (uint64_t)n;
    if (a == b) continue;
    if (a > b) { uint64_t t = a; a = b; b = t; }
    uint64_t key = a * (uint64_t)n + b;
    uint64_t h = mix64(key) & (cap - 1);
    int dup = 0;
    while (table[h] != UINT64_MAX) {
      if (table[h] == key) { dup = 1; break; }
      h = (h + 1) & (cap - 1);
    }
    if (dup) continue;
    table[h] = key;
    src[got] = (int32_t)a;
    dst[got] = (int32_t)b;
    ++got;
  }
  free(table);
  return got;
}

/* ---- CSR assembly ---------------------------------------------------------- */

static int cmp_i32(const void* a, const void* b) {
  int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
  return (x > y) - (x < y);
}

/* Build an n x n CSR pattern from pairs: optional relabelling (perm may be
 * NULL), self-loops dropped, optional symmetrisation (both directions stored),
 * duplicates removed, column indices sorted within each row.
 * rowptr has n+1 entries; colidx needs capacity npairs * (symmetrise ? 2 : 1).
 * Returns nnz, or -1 on allocation failure. */
int64_t synth_build_csr(int64_t n, int64_t npairs, const int32_t* src, const int32_t* dst,
                        const int32_t* perm, int32_t symmetrise,
                        int64_t* rowptr, int32_t* colidx) {
  int64_t* cnt = (int64_t*)calloc((size_t)n + 1, sizeof(int64_t));
  if (!cnt) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < npairs; ++i) {
    int32_t s = src[i], t = dst[i];
    if (s == t) continue;
    if (perm) { s = perm[s]; t = perm[t]; }
#pragma omp atomic
    cnt[s]++;
    if (symmetrise) {
#pragma omp atomic
      cnt[t]++;
    }
  }
  int64_t* start = (int64_t*)malloc(((size_t)n + 1) * sizeof(int64_t));
  int64_t* cursor = (int64_t*)malloc(((size_t)n + 1) * sizeof(int64_t));
  if (!start || !cursor) { free(cnt); free(start); free(cursor); return -1; }
  int64_t total = 0;
  for (int64_t u = 0; u < n; ++u) { start[u] = total; cursor[u] = total; total += cnt[u]; }
  start[n] = total;
  int32_t* raw = (int32_t*)malloc((size_t)(total > 0 ? total : 1) * sizeof(int32_t));
  if (!raw) { free(cnt); free(start); free(cursor); return -1; }
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < npairs; ++i) {
    int32_t s = src[i], t = dst[i];
    if (s == t) continue;
    if (perm) { s = perm[s]; t = perm[t]; }
    int64_t p;
#pragma omp atomic capture
    p = cursor[s]++;
    raw[p] = t;
    if (symmetrise) {
#pragma omp atomic capture
      p = cursor[t]++;
      raw[p] = s;
    }
  }
  /* per-row sort and in-place dedup; cnt[u] becomes the unique count */
#pragma omp parallel for schedule(dynamic, 256)
  for (int64_t u = 0; u < n; ++u) {
    int64_t b = start[u], len = start[u + 1] - b;
    if (len > 1) qsort(raw + b, (size_t)len, sizeof(int32_t), cmp_i32);
    int64_t w = 0;
    for (int64_t k = 0; k < len; ++k) {
      if (k == 0 || raw[b + k] != raw[b + k - 1]) raw[b + w++] = raw[b + k];
    }
    cnt[u] = w;
  }
  int64_t nnz = 0;
  for (int64_t u = 0; u < n; ++u) { rowptr[u] = nnz; nnz += cnt[u]; }
  rowptr[n] = nnz;
#pragma omp parallel for schedule(dynamic, 256)
  for (int64_t u = 0; u < n; ++u) {
    memcpy(colidx + rowptr[u], raw + start[u], (size_t)cnt[u] * sizeof(int32_t));
  }
  free(raw); free(cursor); free(start); free(cnt);
  return nnz;
}

/* Symmetric degree normalisation of an adjacency pattern, the edge weights of
 * a graph-convolution layer: values[e] = 1/sqrt(len(row u) * len(row v)) for
 * e = (u, v), computed in double and rounded once to fp32.  Requires n == m
 * (square pattern).  No self-loops are added. */
void synth_sym_norm_values(int64_t m, const int64_t* rowptr, const int32_t* colidx, float* values) {
#pragma omp parallel for schedule(dynamic, 256)
  for (int64_t u = 0; u < m; ++u) {
    double du = (double)(rowptr[u + 1] - rowptr[u]);
    for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e) {
      int64_t v = colidx[e];
      double dv = (double)(rowptr[v + 1] - rowptr[v]);
      if (dv < 1.0) dv = 1.0;
      values[e] = (float)(1.0 / sqrt(du * dv));
    }
  }
}

int32_t synth_num_threads(void) {
#ifdef _OPENMP
  return (int32_t)omp_get_max_threads();
#else
  return 1;
#endif
}
