/*
 * CPU ORACLE for one pipeline stage of chunk-based pipelined GNN training.
 *
 * TEST INFRASTRUCTURE ONLY.  Slow, plain and written to be checked against the
 * paper by eye.  Nothing in the product path may link, import or call this file;
 * it shares no code, tables or helpers with the HIP library.
 *
 * What it follows
 *   - Algorithm 1, inner loops (chunk k, layer l, vertex v in C_k): AGGREGATE over
 *     neighbours with the current-vs-historical choice, then UPDATE.
 *   - Section 2.1: GCN aggregation = sum over neighbours of h_u / sqrt(D_v D_u);
 *     UPDATE = a fully connected layer (here: + bias, ReLU).
 *   - Section 3.3: V_processed decides which neighbours are read from the current
 *     epoch and which from the historical buffer; C_k joins V_processed BEFORE its
 *     layers run, so the chunk itself (self-loop included) reads current values.
 *   - Section 3.4, technique 3: in the backward pass the gradient that would flow
 *     from a not-yet-processed vertex v back to u is replaced by zero.  The backward
 *     pass walks the chunks in the REVERSE of the forward order; then "processed in
 *     backward" == "read u's current value in forward", and the zero rule gives the
 *     exact gradient of the chunked forward with history held constant.
 *   - Section 3.4, technique 2: update_history copies current levels into the
 *     historical buffers; when it is called is caller policy.
 *   - GCNII variant (formula from the benchmark definition, the paper only cites the
 *     model): p = (1-a) z + a h0 ;  h' = ReLU((1-beta) p + beta p W).
 *   - GraphSage variant (Section 2.1, Equation 1: UPDATE takes both h_v of the previous
 *     layer and z_v; the paper only cites the model, the form is Hamilton et al.'s with
 *     the aggregator's weights given per edge, 1/|N(v)| for the mean aggregator):
 *     h' = ReLU(h_v W_self + z_v W_neigh + b), W stored as [W_self ; W_neigh], 2 d_in x d_out.
 *     v belongs to the chunk being computed, so h_v is its current row.
 *   - ResGCN+ variant (the paper only cites the model; the layer is DeepGCNs' pre-activation
 *     residual block with a GCN convolution): r_u = ReLU(LayerNorm(h_u)), z_v = sum_u A_vu r_u,
 *     h'_v = h_v + z_v W + b.  LayerNorm is over the features of one vertex,
 *     gamma * (x - mean) / sqrt(var + eps) + beta with the biased variance.  The current-vs-historical
 *     choice applies to h_u; the normalisation is this layer's own, so its parameters also receive
 *     gradient through the historical rows (oracle_backward_finish).
 *     Dropout (Section 5 trains with rate 0.5; DeepGCNs' block is Norm -> ReLU -> Dropout -> conv):
 *     r_u = m_u * ReLU(LayerNorm(h_u)), m in {0, 1/(1-p)} per (layer, vertex, feature), the same for every
 *     reader of u in a pass and for u's current and historical row alike.  The mask is a counter-based
 *     draw: SplitMix64 of a per-layer key plus the element's index (oracle_dropout_keep).
 *   - Dropout in GCN and GraphSage layers (Section 5 trains with rate 0.5; the paper does not say where it
 *     sits): on the layer's output, h' = m * ReLU(...), m in {0, 1/(1-p)} per (layer, vertex, feature) with
 *     the same draw.  What is stored - and later read as current or historical embedding - is the value after
 *     dropout, so every reader of a vertex sees the same mask, and it equals dropout on the next layer's
 *     input.  Backward: a positive stored output passed both ReLU and dropout, its gradient is scaled by
 *     1/(1-p).  GCNII layers have no dropout here.
 *
 * Precision: arrays are fp32 storage, every sum runs in fp64.  With quant == 1 the
 * values the GPU path keeps in bf16 (saved aggregation, levels, gradient rows) are
 * rounded to bf16 (round-to-nearest-even) at the moment they are stored, so that
 * ReLU decisions are taken in the same precision on both sides.
 *
 * Parity pins: see tests/test_oracle_pins.py (dense A.H.W, K=1, history==current,
 * first-stage aliasing, a hand-computed 5-vertex example, finite differences,
 * GCNII special cases, push-vs-pull brute force).  No function here is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* storage type of every data array: fp32, or fp64 in the -DORACLE_F64 build that the
 * finite-difference pins use */
#ifdef ORACLE_F64
typedef double real_t;
#else
typedef float real_t;
#endif

typedef struct {
  /* graph: CSR of the normalised adjacency A_hat; row v lists sources u of edges u->v */
  int64_t n;
  const int64_t *row_ptr;
  const int32_t *col;
  const real_t *val;
  /* transposed index (built by oracle_build_transpose): for column u the rows v */
  const int64_t *t_ptr;
  const int32_t *t_row;
  const int64_t *t_edge; /* position of the edge in the CSR arrays (for val) */
  /* chunks: contiguous id ranges */
  int32_t K;
  const int64_t *chunk_ptr;
  const int32_t *chunk_of; /* n entries */
  /* stage */
  int32_t L;
  const int32_t *dims; /* L+1 */
  int32_t variant;     /* 0 GCN, 1 GCNII, 2 GraphSage, 3 ResGCN+ */
  double a;            /* GCNII initial-residual weight */
  const double *beta;  /* GCNII, L entries */
  int32_t quant;       /* 0: fp32 storage, 1: bf16 storage of levels >= 1, Z, dZ, g */
  int32_t level0_f32;  /* with quant: level 0 (and grad_in) stay fp32 */
  real_t *const *W;     /* L arrays d_j x d_{j+1} (GraphSage: 2 d_j x d_{j+1}), row-major */
  real_t *const *b;     /* L arrays d_{j+1} (GCN, GraphSage) */
  real_t *const *cur;   /* L+1 arrays n x d_j */
  real_t *const *hist;  /* L arrays n x d_j */
  const real_t *h0;     /* GCNII: n x d */
  real_t *const *Z;     /* saved aggregation (GCN) or mixed p (GCNII), L arrays n x d_j */
  real_t *const *dZ;    /* L arrays n x d_j */
  double *const *dW;   /* L arrays shaped like W, accumulated (+=) */
  double *const *db;   /* L arrays d_{j+1}, accumulated (+=) */
  double *dH0;         /* GCNII: n x d accumulated (+=) */
  real_t *grad_in;      /* n x d_0 or NULL */
  uint8_t *processed;  /* K flags, forward */
  uint8_t *bprocessed; /* K flags, backward */
  real_t *g0, *g1;      /* scratch: max chunk rows x max d each */
  /* ResGCN+ only */
  real_t *const *ln_g;  /* L arrays d: LayerNorm scale */
  real_t *const *ln_b;  /* L arrays d: LayerNorm shift */
  double *const *d_ln_g; /* accumulated (+=) */
  double *const *d_ln_b;
  double ln_eps;
  int32_t *fwd_pos;     /* K entries: position of every chunk in this pass's forward order */
  int32_t n_fwd;
  double dropout_p;     /* 0: no dropout */
  uint64_t dropout_seed; /* of this pass */
} oracle_stage;

void oracle_set_threads(int n) {
#ifdef _OPENMP
  omp_set_num_threads(n);
#else
  (void)n;
#endif
}

int oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

#ifndef ORACLE_F64
/* bf16 round-to-nearest-even of an fp32 value, returned as fp32 */
static float round_bf16(float x) {
  uint32_t u;
  memcpy(&u, &x, 4);
  if ((u & 0x7F800000u) == 0x7F800000u) return x; /* inf / nan unchanged */
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7FFFu + lsb;
  u &= 0xFFFF0000u;
  memcpy(&x, &u, 4);
  return x;
}
#endif

static inline real_t store(const oracle_stage *s, double x) {
#ifdef ORACLE_F64
  (void)s;
  return x; /* fp64-storage build (finite-difference pins): no rounding at all */
#else
  float f = (float)x;
  return s->quant ? round_bf16(f) : f;
#endif
}

/* grad_in is rounded like the other stored rows unless level 0 is an fp32 buffer */
static inline real_t store_level0(const oracle_stage *s, double x) {
#ifdef ORACLE_F64
  (void)s;
  return x;
#else
  float f = (float)x;
  return (s->quant && !s->level0_f32) ? round_bf16(f) : f;
#endif
}

/* Section 2.1: weight of edge u->v is 1/sqrt(D_v D_u); D = row length of A + I. */
void oracle_gcn_norm(int64_t n, const int64_t *row_ptr, const int32_t *col, real_t *val) {
  for (int64_t v = 0; v < n; ++v) {
    double dv = (double)(row_ptr[v + 1] - row_ptr[v]);
    for (int64_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
      int64_t u = col[e];
      double du = (double)(row_ptr[u + 1] - row_ptr[u]);
      val[e] = (real_t)(1.0 / sqrt(dv * du));
    }
  }
}

/* chunk id of every vertex from the contiguous ranges */
void oracle_chunk_of(int64_t n, int32_t K, const int64_t *chunk_ptr, int32_t *chunk_of) {
  (void)n;
  for (int32_t c = 0; c < K; ++c)
    for (int64_t v = chunk_ptr[c]; v < chunk_ptr[c + 1]; ++v) chunk_of[v] = c;
}

/* Transposed index by counting sort: column u -> (row v, edge position), rows ascending. */
void oracle_build_transpose(int64_t n, const int64_t *row_ptr, const int32_t *col,
                            int64_t *t_ptr, int32_t *t_row, int64_t *t_edge) {
  for (int64_t i = 0; i <= n; ++i) t_ptr[i] = 0;
  for (int64_t e = 0; e < row_ptr[n]; ++e) t_ptr[(int64_t)col[e] + 1]++;
  for (int64_t i = 0; i < n; ++i) t_ptr[i + 1] += t_ptr[i];
  int64_t *pos = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n ? n : 1));
  memcpy(pos, t_ptr, sizeof(int64_t) * (size_t)n);
  for (int64_t v = 0; v < n; ++v)
    for (int64_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
      int64_t p = pos[col[e]]++;
      t_row[p] = (int32_t)v;
      t_edge[p] = e;
    }
  free(pos);
}

void oracle_begin_pass(oracle_stage *s) {
  memset(s->processed, 0, (size_t)s->K);
  memset(s->bprocessed, 0, (size_t)s->K);
  s->n_fwd = 0;
}

/* SplitMix64 output function (Steele, Lea, Flood 2014) */
/* exported so that the test suite can pin this copy of the generator's output function to the published vector */
uint64_t oracle_splitmix64(uint64_t z);
static uint64_t splitmix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

/* 1 if feature c of vertex u survives the dropout of layer j in the pass with this seed.  The layer's key is
 * the generator's output for state seed + (j + 1) * golden; the element's draw is the output for state
 * key + (u * d + c + 1) * golden; its top 24 bits, as a fraction of 2^24, are compared with p. */
uint64_t oracle_splitmix64(uint64_t z) { return splitmix64(z); }

int32_t oracle_dropout_keep(uint64_t seed, int32_t j, int64_t u, int32_t d, int32_t c, double p) {
  const uint64_t golden = 0x9E3779B97F4A7C15ull;
  const uint64_t key = splitmix64(seed + (uint64_t)(j + 1) * golden);
  const uint64_t r = splitmix64(key + (uint64_t)(u * d + c + 1) * golden);
  return (double)(r >> 40) >= p * 16777216.0;
}

/* LayerNorm statistics of one row: mean and 1/sqrt(biased variance + eps) */
static void ln_stats(const real_t *x, int32_t d, double eps, double *mean, double *rstd) {
  double m = 0.0;
  for (int32_t i = 0; i < d; ++i) m += (double)x[i];
  m /= d;
  double var = 0.0;
  for (int32_t i = 0; i < d; ++i) var += ((double)x[i] - m) * ((double)x[i] - m);
  var /= d;
  *mean = m;
  *rstd = 1.0 / sqrt(var + eps);
}

/* r = Dropout(ReLU(LayerNorm(x))) of vertex u, stored like every other row the GPU path keeps */
static void ln_relu_row(const oracle_stage *s, int32_t j, int64_t u, const real_t *x, int32_t d, real_t *r) {
  double mean, rstd;
  ln_stats(x, d, s->ln_eps, &mean, &rstd);
  const double keep_scale = 1.0 / (1.0 - s->dropout_p);
  for (int32_t i = 0; i < d; ++i) {
    double y = (double)s->ln_g[j][i] * (((double)x[i] - mean) * rstd) + (double)s->ln_b[j][i];
    y = y > 0.0 ? y : 0.0;
    if (s->dropout_p > 0.0) y = oracle_dropout_keep(s->dropout_seed, j, u, d, i, s->dropout_p) ? y * keep_scale : 0.0;
    r[i] = store(s, y);
  }
}

/* Backward of r = ReLU(LayerNorm(x)) for one row: dr -> dx (may be NULL), and the parameter gradients. */
static void ln_relu_row_backward(const oracle_stage *s, int32_t j, int64_t u, const real_t *x, int32_t d, const double *dr,
                                 double *dx, double *dg, double *db) {
  double mean, rstd;
  ln_stats(x, d, s->ln_eps, &mean, &rstd);
  double m1 = 0.0, m2 = 0.0;
  double *dxh = (double *)malloc(sizeof(double) * (size_t)d);
  const double keep_scale = 1.0 / (1.0 - s->dropout_p);
  for (int32_t i = 0; i < d; ++i) {
    const double xh = ((double)x[i] - mean) * rstd;
    const double y = (double)s->ln_g[j][i] * xh + (double)s->ln_b[j][i];
    double dn = y > 0.0 ? dr[i] : 0.0; /* ReLU derivative, strict */
    if (s->dropout_p > 0.0) dn = oracle_dropout_keep(s->dropout_seed, j, u, d, i, s->dropout_p) ? dn * keep_scale : 0.0;
    dg[i] += dn * xh;
    db[i] += dn;
    dxh[i] = dn * (double)s->ln_g[j][i];
    m1 += dxh[i];
    m2 += dxh[i] * xh;
  }
  m1 /= d;
  m2 /= d;
  if (dx)
    for (int32_t i = 0; i < d; ++i) {
      const double xh = ((double)x[i] - mean) * rstd;
      dx[i] = rstd * (dxh[i] - m1 - xh * m2);
    }
  free(dxh);
}

/* Integer bookkeeping: how many neighbours of each row of chunk k would be read from
 * the CURRENT buffers if chunk k were aggregated now (processed flags as they stand,
 * with k itself counted as processed). */
void oracle_select_counts(const oracle_stage *s, int32_t k, int32_t *out) {
  for (int64_t v = s->chunk_ptr[k]; v < s->chunk_ptr[k + 1]; ++v) {
    int32_t c = 0;
    for (int64_t e = s->row_ptr[v]; e < s->row_ptr[v + 1]; ++e) {
      int32_t cu = s->chunk_of[s->col[e]];
      if (cu == k || s->processed[cu]) ++c;
    }
    out[v - s->chunk_ptr[k]] = c;
  }
}

/* Algorithm 1, forward: body of the loop over chunks for one chunk k.
 * The caller has already placed level-0 rows of C_k in cur[0]. */
void oracle_forward_chunk(oracle_stage *s, int32_t k) {
  s->processed[k] = 1; /* V_processed <- V_processed U C_k, before the layers */
  if (s->fwd_pos) s->fwd_pos[k] = s->n_fwd++;
  const int64_t v0 = s->chunk_ptr[k], v1 = s->chunk_ptr[k + 1];
  for (int32_t j = 0; j < s->L; ++j) {
    const int32_t din = s->dims[j], dout = s->dims[j + 1];
    const real_t *cur = s->cur[j], *hist = s->hist[j];
    const real_t *W = s->W[j];
#pragma omp parallel
    {
      double *z = (double *)malloc(sizeof(double) * (size_t)din);
      double *y = (double *)malloc(sizeof(double) * (size_t)dout);
      real_t *ru = (real_t *)malloc(sizeof(real_t) * (size_t)din);
#pragma omp for schedule(dynamic, 16)
      for (int64_t v = v0; v < v1; ++v) {
        /* AGGREGATE: processed neighbours -> current epoch, the rest -> history */
        for (int32_t i = 0; i < din; ++i) z[i] = 0.0;
        for (int64_t e = s->row_ptr[v]; e < s->row_ptr[v + 1]; ++e) {
          const int64_t u = s->col[e];
          const real_t *src = s->processed[s->chunk_of[u]] ? cur : hist;
          const double w = (double)s->val[e];
          const real_t *hu = src + u * din;
          if (s->variant == 3) { /* ResGCN+: the neighbour enters normalised and activated */
            ln_relu_row(s, j, u, hu, din, ru);
            hu = ru;
          }
          for (int32_t i = 0; i < din; ++i) z[i] += w * (double)hu[i];
        }
        real_t *zs = s->Z[j] + v * din;
        if (s->variant != 1) {
          for (int32_t i = 0; i < din; ++i) zs[i] = store(s, z[i]);
        } else { /* GCNII initial residual */
          const real_t *h0 = s->h0 + v * din;
          for (int32_t i = 0; i < din; ++i)
            zs[i] = store(s, (1.0 - s->a) * z[i] + s->a * (double)h0[i]);
        }
        /* UPDATE: fully connected layer on the stored aggregation */
        for (int32_t o = 0; o < dout; ++o) y[o] = 0.0;
        const real_t *Wz = s->variant == 2 ? W + (int64_t)din * dout : W; /* GraphSage: the lower half */
        for (int32_t i = 0; i < din; ++i) {
          const double zi = (double)zs[i];
          const real_t *wr = Wz + (int64_t)i * dout;
          for (int32_t o = 0; o < dout; ++o) y[o] += zi * (double)wr[o];
        }
        if (s->variant == 2) { /* GraphSage: the vertex's own previous-level row through W_self */
          const real_t *hv = cur + v * din;
          for (int32_t i = 0; i < din; ++i) {
            const double hi = (double)hv[i];
            const real_t *wr = W + (int64_t)i * dout;
            for (int32_t o = 0; o < dout; ++o) y[o] += hi * (double)wr[o];
          }
        }
        real_t *hn = s->cur[j + 1] + v * dout;
        if (s->variant == 3) { /* ResGCN+: residual, no activation after the convolution */
          const real_t *b = s->b[j];
          const real_t *hv = cur + v * din;
          for (int32_t o = 0; o < dout; ++o) hn[o] = store(s, (double)hv[o] + y[o] + (double)b[o]);
        } else if (s->variant != 1) {
          const real_t *b = s->b[j];
          const double keep_scale = 1.0 / (1.0 - s->dropout_p);
          for (int32_t o = 0; o < dout; ++o) {
            double t = y[o] + (double)b[o];
            t = t > 0.0 ? t : 0.0;
            /* GCN, GraphSage: dropout on the layer's output, i.e. on the embedding every later reader sees */
            if (s->dropout_p > 0.0) t = oracle_dropout_keep(s->dropout_seed, j, v, dout, o, s->dropout_p) ? t * keep_scale : 0.0;
            hn[o] = store(s, t);
          }
        } else { /* GCNII identity mapping: (1-beta) p + beta p W */
          const double be = s->beta[j];
          for (int32_t o = 0; o < dout; ++o) {
            double t = (1.0 - be) * (double)zs[o] + be * y[o];
            hn[o] = store(s, t > 0.0 ? t : 0.0);
          }
        }
      }
      free(z);
      free(y);
      free(ru);
    }
  }
}

/* Backward for chunk k (chunks must come in the reverse of the forward order).
 * grad_out: rows of C_k at level L, (v1-v0) x d_L. */
void oracle_backward_chunk(oracle_stage *s, int32_t k, const real_t *grad_out, int32_t need_input_grad) {
  s->bprocessed[k] = 1;
  const int64_t v0 = s->chunk_ptr[k], v1 = s->chunk_ptr[k + 1], m = v1 - v0;
  real_t *g = s->g0, *gn = s->g1;
  memcpy(g, grad_out, sizeof(real_t) * (size_t)(m * s->dims[s->L]));
  for (int32_t j = s->L - 1; j >= 0; --j) {
    const int32_t din = s->dims[j], dout = s->dims[j + 1];
    const real_t *W = s->W[j];
    const real_t *hn = s->cur[j + 1];
    /* dy = g where the layer's output is positive (ReLU derivative, strict); ResGCN+ has no activation there */
    if (s->variant != 3) {
      /* a positive stored output passed the ReLU and, with dropout, survived it: its gradient carries 1 / (1 - p) */
      const int scaled = s->dropout_p > 0.0 && s->variant != 1;
      const double keep_scale = 1.0 / (1.0 - s->dropout_p);
#pragma omp parallel for schedule(static)
      for (int64_t r = 0; r < m; ++r)
        for (int32_t o = 0; o < dout; ++o) {
          if (!(hn[(v0 + r) * dout + o] > (real_t)0)) g[r * dout + o] = (real_t)0;
          else if (scaled) g[r * dout + o] = store(s, (double)g[r * dout + o] * keep_scale);
        }
    }
    const double wscale = s->variant == 1 ? s->beta[j] : 1.0;
    const int64_t zoff = s->variant == 2 ? (int64_t)din * dout : 0; /* GraphSage: W_neigh is the lower half */
    /* weight gradient: dW[i][o] += scale * sum_v Zsaved[v][i] dy[v][o] */
#pragma omp parallel for schedule(static)
    for (int32_t i = 0; i < din; ++i) {
      double *acc = (double *)calloc((size_t)dout, sizeof(double));
      for (int64_t r = 0; r < m; ++r) {
        const double zi = (double)s->Z[j][(v0 + r) * din + i];
        const real_t *dy = g + r * dout;
        for (int32_t o = 0; o < dout; ++o) acc[o] += zi * (double)dy[o];
      }
      for (int32_t o = 0; o < dout; ++o) s->dW[j][zoff + (int64_t)i * dout + o] += wscale * acc[o];
      free(acc);
    }
    if (s->variant == 2) { /* GraphSage: dW_self[i][o] += sum_v h_v[i] dy[v][o] */
#pragma omp parallel for schedule(static)
      for (int32_t i = 0; i < din; ++i) {
        double *acc = (double *)calloc((size_t)dout, sizeof(double));
        for (int64_t r = 0; r < m; ++r) {
          const double hi = (double)s->cur[j][(v0 + r) * din + i];
          const real_t *dy = g + r * dout;
          for (int32_t o = 0; o < dout; ++o) acc[o] += hi * (double)dy[o];
        }
        for (int32_t o = 0; o < dout; ++o) s->dW[j][(int64_t)i * dout + o] += acc[o];
        free(acc);
      }
    }
    if (s->variant != 1) { /* bias gradient */
      for (int32_t o = 0; o < dout; ++o) {
        double acc = 0.0;
        for (int64_t r = 0; r < m; ++r) acc += (double)g[r * dout + o];
        s->db[j][o] += acc;
      }
    }
    /* gradient w.r.t. the aggregation result */
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < m; ++r) {
      const real_t *dy = g + r * dout;
      real_t *dz = s->dZ[j] + (v0 + r) * din;
      for (int32_t i = 0; i < din; ++i) {
        const real_t *wr = W + zoff + (int64_t)i * dout;
        double acc = 0.0;
        for (int32_t o = 0; o < dout; ++o) acc += (double)dy[o] * (double)wr[o];
        if (s->variant != 1) {
          dz[i] = store(s, acc);
        } else {
          const double be = s->beta[j];
          const double dp = (1.0 - be) * (double)dy[i] + be * acc;
          dz[i] = store(s, (1.0 - s->a) * dp);
          s->dH0[(v0 + r) * din + i] += s->a * dp;
        }
      }
    }
    if (j == 0 && !need_input_grad && s->variant != 3) break; /* ResGCN+: LayerNorm's parameters still need it */
    /* GraphSage: the part of the gradient that reaches h_v directly, through W_self (kept in the scratch
     * rows that receive the next g; v is in the chunk, so this is always a current row) */
    if (s->variant == 2) {
#pragma omp parallel for schedule(static)
      for (int64_t r = 0; r < m; ++r) {
        const real_t *dy = g + r * dout;
        for (int32_t i = 0; i < din; ++i) {
          const real_t *wr = W + (int64_t)i * dout;
          double acc = 0.0;
          for (int32_t o = 0; o < dout; ++o) acc += (double)dy[o] * (double)wr[o];
          gn[r * din + i] = store(s, acc);
        }
      }
    }
    /* transposed aggregation with the zero rule: u in C_k pulls from every v that
     * lists u as a neighbour AND whose chunk has been backward-processed */
#pragma omp parallel
    {
      double *acc = (double *)malloc(sizeof(double) * (size_t)din);
#pragma omp for schedule(dynamic, 16)
      for (int64_t u = v0; u < v1; ++u) {
        for (int32_t i = 0; i < din; ++i) acc[i] = s->variant == 2 ? (double)gn[(u - v0) * din + i] : 0.0;
        for (int64_t p = s->t_ptr[u]; p < s->t_ptr[u + 1]; ++p) {
          const int64_t v = s->t_row[p];
          if (!s->bprocessed[s->chunk_of[v]]) continue; /* technique 3: zeros */
          const double w = (double)s->val[s->t_edge[p]];
          const real_t *dz = s->dZ[j] + v * din;
          for (int32_t i = 0; i < din; ++i) acc[i] += w * (double)dz[i];
        }
        if (s->variant == 3) {
          /* acc is dL/dr_u over the readers that saw u's current row; stored like the GPU's gradient rows,
           * then back through ReLU and LayerNorm of u's own row, plus the residual branch */
          double *dr = (double *)malloc(sizeof(double) * (size_t)din * 2);
          double *dx = dr + din;
          for (int32_t i = 0; i < din; ++i) dr[i] = (double)store(s, acc[i]);
          double *dg = (double *)calloc((size_t)din * 2, sizeof(double));
          ln_relu_row_backward(s, j, u, s->cur[j] + u * din, din, dr, dx, dg, dg + din);
#pragma omp critical
          for (int32_t i = 0; i < din; ++i) {
            s->d_ln_g[j][i] += dg[i];
            s->d_ln_b[j][i] += dg[din + i];
          }
          for (int32_t i = 0; i < din; ++i) acc[i] = (double)g[(u - v0) * dout + i] + dx[i];
          free(dg);
          free(dr);
        }
        if (j == 0) {
          real_t *out = s->grad_in + u * din;
          if (need_input_grad)
            for (int32_t i = 0; i < din; ++i) out[i] = store_level0(s, acc[i]);
        } else {
          real_t *out = gn + (u - v0) * din;
          for (int32_t i = 0; i < din; ++i) out[i] = store(s, acc[i]);
        }
      }
      free(acc);
    }
    real_t *t = g;
    g = gn;
    gn = t;
  }
}

/* ResGCN+ only, after the last backward chunk of a pass.  The historical rows are constants, but the
 * LayerNorm applied to them is this layer's own: its parameters receive gradient through every edge that
 * read u's historical row, i.e. whose reader's chunk came BEFORE u's chunk in the forward order. */
void oracle_backward_finish(oracle_stage *s) {
  if (s->variant != 3) return;
  for (int32_t j = 0; j < s->L; ++j) {
    const int32_t d = s->dims[j];
    double *acc = (double *)malloc(sizeof(double) * (size_t)d * 2);
    double *dr = acc + d;
    for (int64_t u = 0; u < s->n; ++u) {
      const int32_t pu = s->fwd_pos[s->chunk_of[u]];
      for (int32_t i = 0; i < d; ++i) acc[i] = 0.0;
      for (int64_t p = s->t_ptr[u]; p < s->t_ptr[u + 1]; ++p) {
        const int64_t v = s->t_row[p];
        if (s->fwd_pos[s->chunk_of[v]] >= pu) continue; /* that reader saw the current row */
        const double w = (double)s->val[s->t_edge[p]];
        const real_t *dz = s->dZ[j] + v * d;
        for (int32_t i = 0; i < d; ++i) acc[i] += w * (double)dz[i];
      }
      for (int32_t i = 0; i < d; ++i) dr[i] = (double)store(s, acc[i]);
      ln_relu_row_backward(s, j, u, s->hist[j] + u * d, d, dr, NULL, s->d_ln_g[j], s->d_ln_b[j]);
    }
    free(acc);
  }
}

/* Technique 2's copy: historical buffers take the current levels 0..L-1. */
void oracle_update_history(oracle_stage *s) {
  for (int32_t j = 0; j < s->L; ++j)
    if (s->hist[j] != s->cur[j])
      memcpy(s->hist[j], s->cur[j], sizeof(real_t) * (size_t)(s->n * s->dims[j]));
}
