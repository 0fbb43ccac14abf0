/*
 * Seeded synthetic-graph builder (input generator only: it holds none of the
 * GNN method's arithmetic; it produces graph STRUCTURE, never edge weights).
 *
 * R-MAT recursive-quadrant sampling -> undirected simple graph -> optional
 * random relabel -> symmetric CSR with one self-loop per vertex, columns
 * ascending inside every row.  Deterministic for a given (seed, arguments)
 * whatever the thread count: the candidate set is a pure function of the
 * candidate counter, and every row is sorted + deduplicated afterwards.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC rmat_gen.c -o librmat_gen.so
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline uint64_t mix64(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}

/* counter-based 64 random bits for (seed, stream, counter) */
static inline uint64_t rnd64(uint64_t seed, uint64_t stream, uint64_t ctr) {
  return mix64(mix64(seed ^ (stream * 0xD1342543DE82EF95ull)) + ctr);
}

static int cmp_i32(const void *a, const void *b) {
  int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
  return (x > y) - (x < y);
}

/* One R-MAT candidate: `scale` quadrant draws, 16 random bits each. */
static inline void rmat_pair(uint64_t seed, uint64_t i, int scale, uint32_t ta,
                             uint32_t tb, uint32_t tc, int64_t *pu, int64_t *pv) {
  int64_t u = 0, v = 0;
  uint64_t bits = 0;
  for (int l = 0; l < scale; ++l) {
    if ((l & 3) == 0) bits = rnd64(seed, 1 + (uint64_t)(l >> 2), i);
    uint32_t r = (uint32_t)(bits & 0xFFFF);
    bits >>= 16;
    int right = 0, down = 0;
    if (r < ta) { /* top-left */
    } else if (r < tb) {
      right = 1;
    } else if (r < tc) {
      down = 1;
    } else {
      right = 1;
      down = 1;
    }
    u = (u << 1) | down;
    v = (v << 1) | right;
  }
  *pu = u;
  *pv = v;
}

/*
 * Phase 1: returns an opaque handle holding the symmetric CSR; nnz via *out_nnz.
 *   n            vertices (ids >= n drawn from the 2^scale square are rejected)
 *   n_candidates R-MAT draws (duplicates / self pairs / out-of-range are dropped)
 *   a,b,c        quadrant probabilities (d = 1-a-b-c)
 *   relabel      nonzero: apply a seeded random permutation to vertex ids
 * Phase 2: rmat_fill copies row_ptr/col into caller arrays and frees the handle.
 */
typedef struct {
  int64_t n, nnz;
  int64_t *row_ptr;
  int32_t *col;
} rmat_graph;

void *rmat_build(int64_t n, int64_t n_candidates, double a, double b, double c,
                 uint64_t seed, int relabel, int64_t *out_nnz) {
  int scale = 0;
  while (((int64_t)1 << scale) < n) ++scale;
  uint32_t ta = (uint32_t)(a * 65536.0 + 0.5);
  uint32_t tb = ta + (uint32_t)(b * 65536.0 + 0.5);
  uint32_t tc = tb + (uint32_t)(c * 65536.0 + 0.5);

  /* permutation (identity when relabel == 0): Fisher-Yates with counter RNG */
  int32_t *perm = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
  for (int64_t i = 0; i < n; ++i) perm[i] = (int32_t)i;
  if (relabel) {
    for (int64_t i = n - 1; i > 0; --i) {
      uint64_t r = rnd64(seed, 1000, (uint64_t)i) % (uint64_t)(i + 1);
      int32_t t = perm[i];
      perm[i] = perm[r];
      perm[r] = t;
    }
  }

  /* pass A: count candidates per smaller endpoint */
  int64_t *cnt = (int64_t *)calloc((size_t)n + 1, sizeof(int64_t));
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n_candidates; ++i) {
    int64_t u, v;
    rmat_pair(seed, (uint64_t)i, scale, ta, tb, tc, &u, &v);
    if (u >= n || v >= n || u == v) continue;
    int64_t pu = perm[u], pv = perm[v];
    int64_t lo = pu < pv ? pu : pv;
#pragma omp atomic
    cnt[lo + 1]++;
  }
  for (int64_t i = 0; i < n; ++i) cnt[i + 1] += cnt[i];
  int64_t n_valid = cnt[n];
  int32_t *hi_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_valid ? n_valid : 1));
  int64_t *fill = (int64_t *)malloc(sizeof(int64_t) * (size_t)n);
  memcpy(fill, cnt, sizeof(int64_t) * (size_t)n);
  /* pass B: scatter larger endpoint into the bucket of the smaller one */
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n_candidates; ++i) {
    int64_t u, v;
    rmat_pair(seed, (uint64_t)i, scale, ta, tb, tc, &u, &v);
    if (u >= n || v >= n || u == v) continue;
    int64_t pu = perm[u], pv = perm[v];
    int64_t lo = pu < pv ? pu : pv, hi = pu < pv ? pv : pu;
    int64_t slot;
#pragma omp atomic capture
    slot = fill[lo]++;
    hi_of[slot] = (int32_t)hi;
  }
  free(fill);
  free(perm);

  /* sort + dedupe each bucket; uniq[lo] = unique neighbours hi > lo */
  int64_t *uniq = (int64_t *)calloc((size_t)n, sizeof(int64_t));
#pragma omp parallel for schedule(dynamic, 256)
  for (int64_t r = 0; r < n; ++r) {
    int64_t b0 = cnt[r], b1 = cnt[r + 1];
    if (b1 - b0 > 1) qsort(hi_of + b0, (size_t)(b1 - b0), sizeof(int32_t), cmp_i32);
    int64_t w = b0;
    for (int64_t e = b0; e < b1; ++e)
      if (e == b0 || hi_of[e] != hi_of[e - 1]) hi_of[w++] = hi_of[e];
    uniq[r] = w - b0;
  }

  /* degrees of the symmetric graph with self-loops */
  int64_t *deg = (int64_t *)calloc((size_t)n + 1, sizeof(int64_t));
  for (int64_t r = 0; r < n; ++r) {
    deg[r + 1] += uniq[r] + 1; /* +1: self-loop */
    for (int64_t e = cnt[r]; e < cnt[r] + uniq[r]; ++e) deg[(int64_t)hi_of[e] + 1]++;
  }
  for (int64_t i = 0; i < n; ++i) deg[i + 1] += deg[i];
  int64_t nnz = deg[n];
  int32_t *col = (int32_t *)malloc(sizeof(int32_t) * (size_t)nnz);
  int64_t *pos = (int64_t *)malloc(sizeof(int64_t) * (size_t)n);
  memcpy(pos, deg, sizeof(int64_t) * (size_t)n);
  /* Rows are visited in ascending order, so every row receives first its
   * smaller neighbours (ascending), then itself, then its larger ones
   * (ascending): columns come out sorted without another sort. */
  for (int64_t r = 0; r < n; ++r) {
    col[pos[r]++] = (int32_t)r;
    for (int64_t e = cnt[r]; e < cnt[r] + uniq[r]; ++e) {
      int64_t h = hi_of[e];
      col[pos[r]++] = (int32_t)h;
      col[pos[h]++] = (int32_t)r;
    }
  }
  free(pos);
  free(uniq);
  free(hi_of);
  free(cnt);

  rmat_graph *g = (rmat_graph *)malloc(sizeof(rmat_graph));
  g->n = n;
  g->nnz = nnz;
  g->row_ptr = deg;
  g->col = col;
  *out_nnz = nnz;
  return g;
}

void rmat_fill(void *handle, int64_t *row_ptr, int32_t *col) {
  rmat_graph *g = (rmat_graph *)handle;
  memcpy(row_ptr, g->row_ptr, sizeof(int64_t) * (size_t)(g->n + 1));
  memcpy(col, g->col, sizeof(int32_t) * (size_t)g->nnz);
  free(g->row_ptr);
  free(g->col);
  free(g);
}
