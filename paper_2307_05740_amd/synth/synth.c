/*
 * Seeded synthetic inputs for sparse x tall-skinny-dense products: graph
 * patterns (R-MAT, 2-D five-point grid, Chung-Lu power law), nonzero value
 * fills and the dense operand X.
 *
 * This file holds input generation only.  It contains none of the method's
 * arithmetic (no product, no decomposition) and is the one piece of code the
 * test oracle's callers and the GPU library's callers both use.
 *
 * Every random quantity is a pure function of (seed, coordinates) through a
 * counter-based 64-bit mixer, so results do not depend on thread count or
 * scheduling.  The sparse operand is produced in CSR, which is the order-2
 * case of compressed-sparse-fiber storage (paper, section "Tensor Sparsity and
 * Sparse Storage").
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* counter-based generator: the splitmix64 output function applied to  */
/* a key built from the seed and up to two coordinates                 */
/* ------------------------------------------------------------------ */
static inline uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ULL;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
  return z ^ (z >> 31);
}

static inline uint64_t key3(uint64_t seed, uint64_t a, uint64_t b) {
  return mix64(mix64(mix64(seed) ^ a) ^ b);
}

/* ------------------------------------------------------------------ */
/* graph object handed across the C boundary                           */
/* ------------------------------------------------------------------ */
typedef struct synth_graph {
  int64_t n;
  int64_t nnz;
  int64_t *rowptr; /* n + 1 */
  int32_t *colidx; /* nnz, sorted and duplicate-free inside every row */
} synth_graph;

void synth_graph_free(synth_graph *g) {
  if (!g) return;
  free(g->rowptr);
  free(g->colidx);
  free(g);
}

int64_t synth_graph_n(const synth_graph *g) { return g ? g->n : -1; }
int64_t synth_graph_nnz(const synth_graph *g) { return g ? g->nnz : -1; }

/* copy the pattern into caller-owned arrays (rowptr: n+1, colidx: nnz) */
int synth_graph_export(const synth_graph *g, int64_t *rowptr, int32_t *colidx) {
  if (!g || !rowptr || !colidx) return -1;
  memcpy(rowptr, g->rowptr, (size_t)(g->n + 1) * sizeof(int64_t));
  memcpy(colidx, g->colidx, (size_t)g->nnz * sizeof(int32_t));
  return 0;
}

static int cmp_i32(const void *a, const void *b) {
  int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
  return (x > y) - (x < y);
}

/*
 * Directed samples (src[e], dst[e]) -> symmetric pattern: both (u,v) and
 * (v,u) are stored, self loops are kept once, duplicates merge.
 */
static synth_graph *edges_to_symmetric_csr(int64_t n, int64_t m,
                                           const int32_t *src,
                                           const int32_t *dst) {
  synth_graph *g = (synth_graph *)calloc(1, sizeof(*g));
  if (!g) return NULL;
  g->n = n;
  int64_t *cnt = (int64_t *)calloc((size_t)n + 1, sizeof(int64_t));
  if (!cnt) { free(g); return NULL; }

#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < m; ++e) {
    int32_t u = src[e], v = dst[e];
    __atomic_fetch_add(&cnt[u], 1, __ATOMIC_RELAXED);
    if (u != v) __atomic_fetch_add(&cnt[v], 1, __ATOMIC_RELAXED);
  }
  /* exclusive scan into raw row starts */
  int64_t *start = (int64_t *)malloc(((size_t)n + 1) * sizeof(int64_t));
  int64_t *cursor = (int64_t *)malloc(((size_t)n + 1) * sizeof(int64_t));
  if (!start || !cursor) { free(cnt); free(start); free(cursor); free(g); return NULL; }
  int64_t run = 0;
  for (int64_t i = 0; i < n; ++i) { start[i] = run; cursor[i] = run; run += cnt[i]; }
  start[n] = run;
  int32_t *raw = (int32_t *)malloc((size_t)(run > 0 ? run : 1) * sizeof(int32_t));
  if (!raw) { free(cnt); free(start); free(cursor); free(g); return NULL; }

#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < m; ++e) {
    int32_t u = src[e], v = dst[e];
    int64_t p = __atomic_fetch_add(&cursor[u], 1, __ATOMIC_RELAXED);
    raw[p] = v;
    if (u != v) {
      int64_t q = __atomic_fetch_add(&cursor[v], 1, __ATOMIC_RELAXED);
      raw[q] = u;
    }
  }
  free(cursor);

  /* sort every row, drop repeats; cnt[i] becomes the merged length */
#pragma omp parallel for schedule(dynamic, 256)
  for (int64_t i = 0; i < n; ++i) {
    int64_t lo = start[i], len = start[i + 1] - lo;
    if (len > 1) qsort(raw + lo, (size_t)len, sizeof(int32_t), cmp_i32);
    int64_t w = 0;
    for (int64_t p = 0; p < len; ++p)
      if (p == 0 || raw[lo + p] != raw[lo + p - 1]) raw[lo + w++] = raw[lo + p];
    cnt[i] = w;
  }

  g->rowptr = (int64_t *)malloc(((size_t)n + 1) * sizeof(int64_t));
  if (!g->rowptr) { free(cnt); free(start); free(raw); free(g); return NULL; }
  run = 0;
  for (int64_t i = 0; i < n; ++i) { g->rowptr[i] = run; run += cnt[i]; }
  g->rowptr[n] = run;
  g->nnz = run;
  g->colidx = (int32_t *)malloc((size_t)(run > 0 ? run : 1) * sizeof(int32_t));
  if (!g->colidx) { free(cnt); free(start); free(raw); synth_graph_free(g); return NULL; }
#pragma omp parallel for schedule(dynamic, 1024)
  for (int64_t i = 0; i < n; ++i)
    memcpy(g->colidx + g->rowptr[i], raw + start[i], (size_t)cnt[i] * sizeof(int32_t));
  free(cnt); free(start); free(raw);
  return g;
}

/*
 * R-MAT: every sample walks `scale` levels from the most significant bit down
 * and at each level picks a quadrant: (0,0) with probability a, (0,1) with b,
 * (1,0) with c, (1,1) with d; the first bit goes to the row, the second to the
 * column.  No noise, no label scrambling.  n = 2^scale, `samples` directed
 * samples, then symmetrised with duplicates merged.
 */
synth_graph *synth_rmat(int32_t scale, int64_t samples, double a, double b,
                        double c, uint64_t seed) {
  if (scale < 1 || scale > 30 || samples < 0) return NULL;
  int64_t n = (int64_t)1 << scale;
  int32_t *src = (int32_t *)malloc((size_t)(samples > 0 ? samples : 1) * sizeof(int32_t));
  int32_t *dst = (int32_t *)malloc((size_t)(samples > 0 ? samples : 1) * sizeof(int32_t));
  if (!src || !dst) { free(src); free(dst); return NULL; }
  const double two32 = 4294967296.0;
  const uint32_t ta = (uint32_t)(a * two32);
  const uint32_t tab = (uint32_t)((a + b) * two32);
  const uint32_t tabc = (uint32_t)((a + b + c) * two32);
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < samples; ++e) {
    uint32_t u = 0, v = 0;
    uint64_t bits = 0;
    for (int32_t l = 0; l < scale; ++l) {
      if ((l & 1) == 0) bits = key3(seed, (uint64_t)e, (uint64_t)(l >> 1));
      uint32_t r = (uint32_t)(bits & 0xFFFFFFFFu);
      bits >>= 32;
      uint32_t rb = (r >= tab) ? 1u : 0u;                  /* row bit    */
      uint32_t cb = (r >= ta && r < tab) || (r >= tabc);   /* column bit */
      u = (u << 1) | rb;
      v = (v << 1) | cb;
    }
    src[e] = (int32_t)u;
    dst[e] = (int32_t)v;
  }
  synth_graph *g = edges_to_symmetric_csr(n, samples, src, dst);
  free(src); free(dst);
  return g;
}

/*
 * Chung-Lu: vertex v carries weight w_v proportional to (v+1)^(-1/(gamma-1)),
 * scaled to mean `avg_deg`, clipped at `max_deg` and rescaled to the mean
 * again; both endpoints of each of n*avg_deg/2 samples are drawn independently
 * with probability proportional to w.  Symmetrised, duplicates merged.
 */
synth_graph *synth_chung_lu(int64_t n, double gamma, double avg_deg,
                            double max_deg, uint64_t seed) {
  if (n < 1 || n > 2147483647LL || gamma <= 1.0 || avg_deg <= 0.0) return NULL;
  double *cum = (double *)malloc(((size_t)n + 1) * sizeof(double));
  if (!cum) return NULL;
  const double ex = -1.0 / (gamma - 1.0);
  double tot = 0.0;
  for (int64_t v = 0; v < n; ++v) { cum[v + 1] = pow((double)(v + 1), ex); tot += cum[v + 1]; }
  /* two rounds of scale-to-mean, clip */
  for (int round = 0; round < 2; ++round) {
    double s = avg_deg * (double)n / tot;
    tot = 0.0;
    for (int64_t v = 0; v < n; ++v) {
      double w = cum[v + 1] * s;
      if (round == 0 && w > max_deg) w = max_deg;
      cum[v + 1] = w;
      tot += w;
    }
  }
  cum[0] = 0.0;
  for (int64_t v = 0; v < n; ++v) cum[v + 1] += cum[v];
  const double total = cum[n];
  int64_t samples = (int64_t)(avg_deg * (double)n / 2.0);
  int32_t *src = (int32_t *)malloc((size_t)(samples > 0 ? samples : 1) * sizeof(int32_t));
  int32_t *dst = (int32_t *)malloc((size_t)(samples > 0 ? samples : 1) * sizeof(int32_t));
  if (!src || !dst) { free(src); free(dst); free(cum); return NULL; }
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < samples; ++e) {
    int32_t end[2];
    for (int s = 0; s < 2; ++s) {
      uint64_t h = key3(seed, (uint64_t)e, (uint64_t)s);
      double t = (double)(h >> 11) * (1.0 / 9007199254740992.0) * total;
      /* first v with cum[v+1] > t */
      int64_t lo = 0, hi = n - 1;
      while (lo < hi) {
        int64_t mid = (lo + hi) >> 1;
        if (cum[mid + 1] > t) hi = mid; else lo = mid + 1;
      }
      end[s] = (int32_t)lo;
    }
    src[e] = end[0];
    dst[e] = end[1];
  }
  free(cum);
  synth_graph *g = edges_to_symmetric_csr(n, samples, src, dst);
  free(src); free(dst);
  return g;
}

/*
 * Five-point stencil on an N x N grid, vertex id = y*N + x (natural order),
 * no wrap-around: the pattern holds the diagonal and the up-to-four grid
 * neighbours of every vertex.
 */
synth_graph *synth_grid5(int64_t N) {
  if (N < 1 || N > 46340) return NULL;
  synth_graph *g = (synth_graph *)calloc(1, sizeof(*g));
  if (!g) return NULL;
  int64_t n = N * N;
  g->n = n;
  g->rowptr = (int64_t *)malloc(((size_t)n + 1) * sizeof(int64_t));
  if (!g->rowptr) { free(g); return NULL; }
  int64_t run = 0;
  for (int64_t y = 0; y < N; ++y)
    for (int64_t x = 0; x < N; ++x) {
      g->rowptr[y * N + x] = run;
      run += 1 + (y > 0) + (y < N - 1) + (x > 0) + (x < N - 1);
    }
  g->rowptr[n] = run;
  g->nnz = run;
  g->colidx = (int32_t *)malloc((size_t)run * sizeof(int32_t));
  if (!g->colidx) { synth_graph_free(g); return NULL; }
#pragma omp parallel for schedule(static)
  for (int64_t y = 0; y < N; ++y)
    for (int64_t x = 0; x < N; ++x) {
      int64_t i = y * N + x, p = g->rowptr[i];
      if (y > 0) g->colidx[p++] = (int32_t)(i - N);
      if (x > 0) g->colidx[p++] = (int32_t)(i - 1);
      g->colidx[p++] = (int32_t)i;
      if (x < N - 1) g->colidx[p++] = (int32_t)(i + 1);
      if (y < N - 1) g->colidx[p++] = (int32_t)(i + N);
    }
  return g;
}

/* ------------------------------------------------------------------ */
/* value fills (caller-owned CSR arrays)                               */
/* ------------------------------------------------------------------ */

/* independent uniform values on [-1, 1): 24 random bits per stored entry,
 * keyed by (seed, row, column); every value is exact in fp32 */
int synth_fill_uniform(int64_t n, const int64_t *rowptr, const int32_t *colidx,
                       uint64_t seed, float *vals) {
  if (n < 0 || !rowptr || !colidx || !vals) return -1;
#pragma omp parallel for schedule(dynamic, 1024)
  for (int64_t i = 0; i < n; ++i)
    for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
      uint64_t h = key3(seed, (uint64_t)i, (uint64_t)colidx[p]);
      vals[p] = (float)((double)(h >> 40) * (1.0 / 8388608.0) - 1.0);
    }
  return 0;
}

/* random-walk normalisation: every stored entry of row i is 1/len(row i) */
int synth_fill_row_normalized(int64_t n, const int64_t *rowptr, float *vals) {
  if (n < 0 || !rowptr || !vals) return -1;
#pragma omp parallel for schedule(dynamic, 1024)
  for (int64_t i = 0; i < n; ++i) {
    int64_t len = rowptr[i + 1] - rowptr[i];
    float w = len > 0 ? (float)(1.0 / (double)len) : 0.0f;
    for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) vals[p] = w;
  }
  return 0;
}

/* grid operator values: 4 on the diagonal, -1 on every neighbour entry */
int synth_fill_grid5(int64_t n, const int64_t *rowptr, const int32_t *colidx,
                     float *vals) {
  if (n < 0 || !rowptr || !colidx || !vals) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i)
    for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p)
      vals[p] = (colidx[p] == i) ? 4.0f : -1.0f;
  return 0;
}

/* ------------------------------------------------------------------ */
/* dense operand: n x k, row-major, standard normal by Box-Muller on    */
/* two uniforms keyed by (seed, row, column pair)                       */
/* ------------------------------------------------------------------ */
int synth_normal_matrix(int64_t n, int32_t k, uint64_t seed, float *X) {
  if (n < 0 || k < 1 || !X) return -1;
  const double two_pi = 6.283185307179586476925286766559;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    float *row = X + i * (int64_t)k;
    for (int32_t c = 0; c < k; c += 2) {
      uint64_t h1 = key3(seed, (uint64_t)i, (uint64_t)c);
      uint64_t h2 = mix64(h1);
      double u1 = ((double)(h1 >> 11) + 1.0) * (1.0 / 9007199254740992.0); /* (0,1] */
      double u2 = (double)(h2 >> 11) * (1.0 / 9007199254740992.0);         /* [0,1) */
      double r = sqrt(-2.0 * log(u1));
      row[c] = (float)(r * cos(two_pi * u2));
      if (c + 1 < k) row[c + 1] = (float)(r * sin(two_pi * u2));
    }
  }
  return 0;
}

int synth_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
