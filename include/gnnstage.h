/*
 * gnnstage — one pipeline stage of chunk-based pipelined full-graph GNN training on one
 * MI355X (gfx950).  C ABI; no C++ or framework types cross this boundary.
 *
 * The stage owns L consecutive GNN layers and sweeps the whole graph chunk by chunk
 * (Algorithm 1 of the paper, the loops over k, l and v in C_k).  For every destination
 * row v of the chunk it aggregates the CSR neighbours u through the normalised adjacency,
 * reading the CURRENT level-(l-1) row of u when u's chunk has already been started in this
 * pass and the HISTORICAL row otherwise (Section 3.3), then applies the layer's dense
 * update.  The backward pass walks the chunks in the reverse order and drops the gradient
 * that would flow back from a not-yet-processed vertex (Section 3.4, third technique).
 *
 * Level j (0 <= j <= L) is the embedding after j of the stage's layers; level 0 is the
 * stage input.  d_j = dims[j] is its width.  All matrices are dense row-major with
 * leading dimension equal to their width.
 *
 * Pointers are tagged HOST or DEVICE below.  Everything the descriptor points to stays
 * owned by the caller; DEVICE buffers must outlive the handle, HOST arrays are copied by
 * gnnstage_create and may be freed afterwards.  The library allocates no device memory:
 * all of its own device state lives in the caller-provided workspace.
 *
 * Every function returns GNNSTAGE_OK (0) or a negative GNNSTAGE_E* code and never throws
 * or aborts; gnnstage_last_error gives a message for the last failure.
 *
 * stage_forward_chunk, stage_backward_chunk, update_history and gnnstage_flush_weight_gradients do nothing on the
 * device but launch kernels on the given stream (no allocation, no synchronisation, no memset or copy call), so with
 * the gnnstage_profile_* timers off a sequence of them may be recorded under HIP stream capture and replayed; the
 * protocol state they keep on the host (which chunks are processed) advances at capture time, so a replay repeats
 * exactly the recorded calls.
 */
#ifndef GNNSTAGE_H
#define GNNSTAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gnnstage gnnstage_t; /* opaque, owned by the library */

enum {
  GNNSTAGE_OK = 0,
  GNNSTAGE_EINVAL = -1,  /* null pointer, bad shape / dtype / variant, malformed CSR or chunks */
  GNNSTAGE_ERANGE = -2,  /* chunk id outside [0, n_chunks) */
  GNNSTAGE_EORDER = -3,  /* call sequence violates the pass protocol (see below) */
  GNNSTAGE_ENOMEM = -4,  /* workspace smaller than gnnstage_workspace_size(), or the host ran out of memory */
  GNNSTAGE_EHIP = -5,    /* a HIP runtime call failed */
  GNNSTAGE_ENOTSUP = -6  /* sizes beyond what the index packing supports */
};

enum { GNNSTAGE_GCN = 0, GNNSTAGE_GCNII = 1, GNNSTAGE_SAGE = 2, GNNSTAGE_RESGCN = 3 };
enum { GNNSTAGE_F32 = 0, GNNSTAGE_BF16 = 1 };

/*
 * Stage descriptor (the inputs of Algorithm 1 for one GPU: graph, chunks, the layers
 * assigned to this GPU and their weights, plus the embedding buffers).
 *
 * variant GNNSTAGE_GCN   (Section 2.1):  z_v = sum_u A_vu src(u);  h'_v = ReLU(z_v W + b)
 * variant GNNSTAGE_GCNII (benchmark definition; the paper only cites the model):
 *     p_v = (1-alpha) z_v + alpha h0_v ;  h'_v = ReLU((1-beta_l) p_v + beta_l p_v W)
 *     (all widths equal, no bias).
 * variant GNNSTAGE_SAGE  (Section 2.1, Equation 1: UPDATE takes h_v of the previous layer and z_v; the
 *     paper only cites the model, the form is Hamilton et al.'s):
 *     h'_v = ReLU(h_v W_self + z_v W_neigh + b), W[j] = [W_self ; W_neigh] stacked, 2 d_j x d_{j+1}
 *     (dW[j] likewise).  v is in the chunk being computed, so h_v is its current row.  The aggregator's
 *     weights are edge_val; edge_val == NULL means the mean aggregator, 1 / (length of row v).
 * variant GNNSTAGE_RESGCN (the paper only cites the model; DeepGCNs' pre-activation residual block with a
 *     GCN convolution):  r_u = ReLU(LayerNorm_j(h_u)),  z_v = sum_u A_vu r_u,  h'_v = h_v + z_v W + b.
 *     LayerNorm over the features of one vertex, gamma * (x - mean) / sqrt(var + ln_eps) + beta with the biased
 *     variance.  The current-vs-historical choice applies to h_u.  All widths equal (at most 1024), no fp32
 *     level 0.  d_ln_gamma / d_ln_beta are complete after the last backward call of a pass: the normalisation
 *     is the layer's own, so its parameters also receive gradient through the historical rows.
 *     With dropout_p > 0 (Section 5 trains with rate 0.5) the block is Norm -> ReLU -> Dropout -> convolution:
 *     r_u is zeroed or scaled by 1 / (1 - p) per (layer, vertex, feature), the same decision for every reader
 *     of u in a pass and for u's current and historical row; decisions are counter-based draws from the seed
 *     given by gnnstage_set_dropout_seed.
 * Dropout in GNNSTAGE_GCN and GNNSTAGE_SAGE stages (dropout_p > 0; Section 5 trains with rate 0.5, the paper does
 *     not say where it sits): on the output of every layer of the stage, h' = m * ReLU(...), m in {0, 1/(1-p)}
 *     per (layer, vertex, feature) from the same draws.  What the level buffers hold - and what later readers
 *     gather as current or historical embedding - is the value after dropout, which equals dropout on the next
 *     layer's input with one mask for all readers of a vertex.  Backward: a positive stored output passed ReLU and
 *     dropout, its gradient is scaled by 1 / (1 - p).  A stage whose last layer is the model's output layer should
 *     be created with dropout_p = 0.  GNNSTAGE_GCNII takes no dropout (EINVAL).
 *
 * dtype GNNSTAGE_F32 : levels, weights, gradients rows are fp32; fp32 arithmetic.
 * dtype GNNSTAGE_BF16: levels, weights, gradient rows are bf16 (bias and all accumulators
 *     fp32; products on the bf16 matrix cores with fp32 accumulation).  With level0_f32 != 0
 *     level 0 (cur[0], hist[0], grad_in) is fp32 instead (a first stage fed with raw features).
 */
typedef struct {
  /* graph: CSR of A_hat INCLUDING self-loops; row v lists the sources u of edges u->v (any
   * order inside a row, no symmetry assumed).  HOST. */
  int64_t n_vertices;
  int64_t nnz;
  const int64_t *row_ptr; /* HOST, n_vertices + 1 */
  const int32_t *col_idx; /* HOST, nnz */
  const float *edge_val;  /* HOST, nnz; NULL => 1/sqrt(D_v D_u), D = row length (Section 2.1) */
  /* chunks: chunk c = vertex ids [chunk_ptr[c], chunk_ptr[c+1]); empty chunks allowed */
  int32_t n_chunks;
  const int64_t *chunk_ptr; /* HOST, n_chunks + 1, chunk_ptr[0] = 0, last = n_vertices */
  /* layers */
  int32_t n_layers;
  const int32_t *dims; /* HOST, n_layers + 1 */
  int32_t variant;
  float alpha;       /* GCNII initial-residual weight */
  const float *beta; /* HOST, n_layers; GCNII only (NULL for GCN) */
  int32_t dtype;
  int32_t level0_f32;
  /* HOST arrays of DEVICE pointers */
  void *const *W;      /* n_layers; W[j] is d_j x d_{j+1}; read when a pass starts (forward) and
                          at each backward call; must not change inside a pass */
  void *const *bias;   /* n_layers fp32 vectors d_{j+1}; GCN only (NULL for GCNII) */
  void *const *cur;    /* n_layers + 1; n x d_j.  The caller fills level-0 rows of chunk c before
                          stage_forward_chunk(c); the library writes rows of c at levels 1..L */
  void *const *hist;   /* n_layers (levels 0..L-1); hist[0] may alias cur[0] (first stage) */
  const void *h0;      /* DEVICE n x d, GCNII only */
  float *const *dW;    /* n_layers fp32 d_j x d_{j+1}; "+=" over the backward calls; caller zeroes */
  float *const *dbias; /* n_layers fp32 d_{j+1}; "+="; GCN only */
  void *grad_in;       /* DEVICE n x d_0 (level-0 dtype); rows of chunk c written by its backward
                          call; used only when need_input_grad != 0 */
  float *grad_h0;      /* DEVICE fp32 n x d, "+="; GCNII only */
  int32_t need_input_grad;
  void *workspace;     /* DEVICE, 256-byte aligned, >= gnnstage_workspace_size() bytes */
  size_t workspace_bytes;
  /* GNNSTAGE_RESGCN only: HOST arrays (n_layers) of DEVICE fp32 vectors of width d_j */
  void *const *ln_gamma;
  void *const *ln_beta;
  float *const *d_ln_gamma; /* "+=" over the backward calls; caller zeroes */
  float *const *d_ln_beta;
  float ln_eps;
  float dropout_p; /* in [0, 1), 0 = none.  GNNSTAGE_RESGCN: between ReLU and the convolution; GNNSTAGE_GCN,
                      GNNSTAGE_SAGE: on every layer's output; GNNSTAGE_GCNII: must be 0 */
} gnnstage_desc;

/* Device bytes the stage needs inside desc->workspace (graph tables, transposed index,
 * launch schedule, saved aggregations for backward, gradient rows).  Host-only computation;
 * returns 0 when the descriptor's sizes are invalid.  Reads row_ptr, col_idx, chunk_ptr and
 * dims; no other pointer field is dereferenced. */
size_t gnnstage_workspace_size(const gnnstage_desc *desc);

/* Validates the descriptor, builds the transposed (CSC) index and the launch schedule on the
 * host, uploads them into the workspace and synchronises.  *out is NULL on failure. */
int gnnstage_create(const gnnstage_desc *desc, gnnstage_t **out);

/*
 * Forward work of one chunk: Algorithm 1, the body of the loop over k for this GPU's layers.
 * pos_in_pass is the position of the chunk in this pass's processing order: 0 starts a new
 * pass (V_processed <- empty) and the following calls must use 1, 2, ... with every chunk at
 * most once (any permutation: Section 3.4 chunk shuffling).  The chunk counts as processed
 * for its own aggregation.  Asynchronous on hip_stream (a hipStream_t; NULL = default stream).
 * Errors: ERANGE (chunk id), EORDER (pos out of sequence, chunk seen twice).
 */
int stage_forward_chunk(gnnstage_t *st, int32_t chunk_id, int32_t pos_in_pass, void *hip_stream);

/*
 * Backward work of one chunk.  grad_out_rows: DEVICE, rows of the chunk at level L,
 * (chunk rows) x d_L, level dtype.  Chunks must come in exactly the reverse of the forward
 * order of a completed forward pass (otherwise EORDER): then a vertex is "processed" in the
 * backward pass exactly when it read current values in the forward pass, and the zero rule of
 * Section 3.4 yields the gradient of the chunked forward with history held constant.
 * Accumulates dW, dbias (and grad_h0), writes grad_in rows of the chunk when requested.  dW and dbias are complete
 * after the last backward call of the pass (see gnnstage_flush_weight_gradients).
 */
int stage_backward_chunk(gnnstage_t *st, int32_t chunk_id, const void *grad_out_rows, void *hip_stream);

/* The library takes the weight gradient of a layer in ONE product over all rows once the backward pass is complete
 * (the last stage_backward_chunk call of a pass does it), not chunk by chunk.  A caller that stops a backward pass
 * early calls this to have dW / dbias hold the contributions of the backward calls made so far; it is a no-op when
 * nothing is owed.  (Layers that run transform-first owe a further term that needs every chunk's gradient rows;
 * their dW is complete only after the last backward call.)  Asynchronous on hip_stream. */
int gnnstage_flush_weight_gradients(gnnstage_t *st, void *hip_stream);

/* hist[j] <- cur[j] for j < L, all rows (Section 3.4, second technique: when to call it, i.e.
 * the refresh period, is caller policy).  Levels whose hist pointer aliases cur are skipped. */
int update_history(gnnstage_t *st, void *hip_stream);

/* The same refresh without moving a byte, for callers that let the library say which buffer is which (Section 3.4,
 * second technique, at a refresh period of one epoch).  For every level j in [1, L) whose hist pointer differs from
 * its cur pointer the two buffers trade places INSIDE the library: the buffer that held the current level becomes
 * the historical one, and the next pass writes its current rows into the other buffer.  That is the state
 * update_history leaves, except that the new "current" buffer holds stale rows: harmless, because a pass reads a
 * current row only after it has written it (rows of processed chunks), and everything else from history.  Level 0 is
 * caller-filled and keeps its buffers: it is copied as in update_history when hist[0] differs from cur[0].
 * Needs a complete pass behind it (every chunk forwarded; no backward pass half-way), otherwise EORDER.
 * After the call gnnstage_level_buffers tells where the levels are; the desc's pointers no longer do. */
int gnnstage_update_history_swap(gnnstage_t *st, void *hip_stream);

/* Where level `level` lives now: *cur (levels 0 .. L) and *hist (levels 0 .. L-1, NULL for level L), DEVICE pointers
 * among those the caller passed at create.  Either output may be NULL.  EINVAL for a level outside [0, L]. */
int gnnstage_level_buffers(const gnnstage_t *st, int32_t level, void **cur, void **hist);

/* Seed of the dropout decisions of the passes that follow.  Feature c of vertex u survives in layer j when the
 * top 24 bits of SplitMix64(key_j + (u * d + c + 1) * G) are at least dropout_p * 2^24, key_j = SplitMix64(seed +
 * (j + 1) * G), G = 0x9E3779B97F4A7C15, d the width of the rows the dropout acts on (the layer's input for
 * GNNSTAGE_RESGCN, its output for GNNSTAGE_GCN / GNNSTAGE_SAGE).  A pass takes the seed (and the rate) that are
 * set when its first forward call arrives and keeps them until its last backward call, so the backward pass
 * redraws the decisions of its own forward pass even if the caller sets a new seed in between.  EORDER inside a
 * forward or a backward pass. */
int gnnstage_set_dropout_seed(gnnstage_t *st, uint64_t seed);

/* Changes dropout_p for the passes that follow (Section 5 evaluates the trained model: a forward pass with
 * rate 0, then training goes on with the old rate).  Taken by a pass at its first forward call, like the seed.
 * EORDER inside a forward or a backward pass, EINVAL outside [0, 1) or for a positive rate on a GNNSTAGE_GCNII
 * stage. */
int gnnstage_set_dropout_rate(gnnstage_t *st, float dropout_p);

/* Synchronises the device and frees the handle (the workspace stays with the caller). */
int gnnstage_destroy(gnnstage_t *st);

/* Message for the last error on this handle (or, with NULL, of the last failed create). */
const char *gnnstage_last_error(const gnnstage_t *st);

/*
 * Diagnostics for bit-exact tests of the V_processed bookkeeping (Section 3.3): for every row
 * of the chunk, the number of neighbours that WOULD be read from the current buffers if the
 * chunk were aggregated now (processed set as it stands, the chunk itself included).  Pure
 * host computation on the library's own packed tables.  out: HOST, chunk rows.
 */
int gnnstage_debug_select_counts(gnnstage_t *st, int32_t chunk_id, int32_t *out);

/*
 * Order in which layer j (0 <= j < L) applies its two steps: 0 = aggregate, then transform (the order
 * Algorithm 1 prints); 1 = transform, then aggregate.  Both compute A_hat H W with the same per-edge
 * current/history choice; the library transforms first when that narrows the rows the aggregation
 * gathers (d_{j+1} * element size < d_j * element size), GCN layers only.  Negative on error.
 */
int gnnstage_layer_order(const gnnstage_t *st, int32_t layer);

/* What the handle was created with (for code that chains stages: the training loop in gnntrain.h).
 * gnnstage_query returns a shape value, index being the level for WIDTH and the chunk boundary for
 * CHUNK_PTR (negative on error); gnnstage_buffer returns one of the caller's DEVICE buffers (cur[index],
 * hist[index], or grad_in, which is NULL unless need_input_grad was set). */
enum {
  GNNSTAGE_Q_VERTICES = 0, GNNSTAGE_Q_CHUNKS = 1, GNNSTAGE_Q_LAYERS = 2, GNNSTAGE_Q_DTYPE = 3,
  GNNSTAGE_Q_LEVEL0_F32 = 4, GNNSTAGE_Q_VARIANT = 5, GNNSTAGE_Q_NEED_INPUT_GRAD = 6, GNNSTAGE_Q_WIDTH = 7,
  GNNSTAGE_Q_CHUNK_PTR = 8
};
enum { GNNSTAGE_B_CUR = 0, GNNSTAGE_B_HIST = 1, GNNSTAGE_B_GRAD_IN = 2 };
int64_t gnnstage_query(const gnnstage_t *st, int32_t what, int32_t index);
void *gnnstage_buffer(const gnnstage_t *st, int32_t which, int32_t index);

/* Diagnostics: how many entries of the (transposed != 0: transposed) index are multiplied as dense blocks
 * (see gnnstage_dense_plan_create below); 0 when the stage does not use them. */
int64_t gnnstage_dense_entries(const gnnstage_t *st, int32_t transposed);

/*
 * Host-only planning helpers (no GPU needed), exported so that the integer bookkeeping can be
 * checked on a CPU: the transposed index (column u -> rows v ascending, with the position of
 * each entry in the CSR arrays) and the packed column words (vertex id | chunk id << vbits).
 */
int gnnstage_plan_transpose(int64_t n, const int64_t *row_ptr, const int32_t *col_idx,
                            int64_t *t_ptr, int32_t *t_row, int64_t *t_edge);
int gnnstage_plan_pack(int64_t n, int64_t nnz, const int32_t *idx, int32_t n_chunks,
                       const int64_t *chunk_ptr, uint32_t *packed, int32_t *vbits);
/* Launch schedule of one aggregation over rows [row_begin, row_end) of a sparse index (ptr, idx).
 * A task is what one wavefront does.  Rows with at most split_edges entries are one task each
 * (task_slot = -1).  Longer rows are cut into pieces of at most split_edges entries; with n_classes > 1
 * rows of at least class_min_row entries are first cut where the source id changes its range class
 * (class q = source ids [class_lo[q], class_lo[q + 1]), n_classes + 1 ascending bounds from 0 to at most
 * n_vertices - ids from class_lo[n_classes] on belong to no class and their run is cut into class-less pieces;
 * class_lo == NULL means equal id ranges up to n_vertices), so that each piece gathers from one slice of the
 * source table.  (The stage also calls this with `idx` holding, instead of ids, the hotness RANK of every
 * entry's source, ascending inside a row: classes are then slices of the most often gathered sources.)  Every piece carries the index of the fp32 partial-sum slot it writes (consecutive per row).
 * force_slot (one byte per vertex, may be NULL) marks rows whose sum has parts outside this index: such a row
 * always writes partial sums (never the finished row), and gets no task at all when it is empty here.
 * Tasks are emitted class-major: the pieces of class 0, ..., class n_classes-1 (inside a class the longest
 * piece first, ties in row order), then pieces without a class, then whole rows (both in row order); class_off (n_classes + 1 entries, may be NULL) receives where each class
 * section starts (the last entry is the start of the class-less tail) and slot_class (one byte per slot,
 * may be NULL) the class of every slot (255 = none).  Returns the number of tasks (or a negative code);
 * with non-NULL task arrays also fills them (capacity checked).  idx may be NULL when n_classes == 1. */
int64_t gnnstage_plan_tasks(const int64_t *ptr, const int32_t *idx, int64_t n_vertices, int64_t row_begin,
                            int64_t row_end, int32_t split_edges, int32_t n_classes, const int64_t *class_lo,
                            int32_t class_min_row, const uint8_t *force_slot, int64_t capacity, int32_t *task_row,
                            int64_t *task_e0, int32_t *task_ne, int32_t *task_slot, int64_t *n_slots,
                            int64_t *class_off, uint8_t *slot_class);

/*
 * Chunk partitioner (host only): Algorithm 1's first step, "partition V into K chunks", locality-aware as
 * Section 3.3 asks.  Restreaming FENNEL (Tsourakakis et al., WSDM 2014; Nishimura and Ugander, KDD 2013):
 * `passes` streams over the vertices in index order; a vertex leaves its part, then joins the part i that
 * maximises  |N(v) in P_i| - alpha * 1.5 * sqrt(|P_i|)  among the parts with fewer than ceil(slack * n / K)
 * vertices, alpha = balance * sqrt(K) * m / n^1.5 with m the number of undirected edges (balance = 1 is the
 * published weight, 4 keeps the capacity from binding while the parts form); ties go to the lowest part;
 * self-loops are ignored.  The index must be symmetric for the edge count to mean what it says.
 * by_entries != 0 counts balance in entries of the index (what a chunk costs to aggregate) instead of vertices:
 * vertex v weighs its row length, n becomes the total weight in alpha and in the capacity, and v's balance term
 * is multiplied by its weight; a part is open while it is below the capacity.
 * part (n): part of every vertex.  perm (n): perm[old id] = new id, part by part, index order kept inside a
 * part.  chunk_ptr (K + 1): the id ranges of the chunks after the renumbering.  gnnstage_permute_csr applies a
 * renumbering to an index (columns ascending inside every row).
 * All arrays are HOST memory owned by the caller.  GNNSTAGE_EINVAL for NULL arrays, n < 1, n_chunks < 1, passes < 1,
 * slack < 1, balance < 0, an index entry outside [0, n), or by_entries on an index without entries.  Parts may stay
 * empty (chunks of no vertices), e.g. when n_chunks > n.
 */
int gnnstage_partition_chunks(int64_t n, const int64_t *row_ptr, const int32_t *col_idx, int32_t n_chunks,
                              int32_t passes, double slack, double balance, int32_t by_entries, int32_t *part,
                              int32_t *perm, int64_t *chunk_ptr);
int gnnstage_permute_csr(int64_t n, const int64_t *row_ptr, const int32_t *col_idx, const int32_t *perm,
                         int64_t *out_ptr, int32_t *out_idx);

/* Dense-block plan of one aggregation direction (host only).  Power-law graphs keep most of their
 * entries in a small, dense corner once rows and columns are ordered by degree: inside every chunk the
 * rows are ordered by length, the vertices of every chunk by how often they occur as a column, and the
 * matrix is cut into blocks of 128 rows x 64 columns in those orders.  Blocks with at least min_nnz
 * entries are multiplied as dense tiles on the matrix cores; their entries leave the sparse index (the
 * "remainder", same rows, same column order).  If fewer than min_share of all entries fall into such
 * blocks the plan stays inactive (every array below empty).  gnnstage_dense_plan_get returns the length
 * of one array of the plan and a pointer to it (valid until destroy):
 *   0 rem_ptr (int64, n+1)   1 rem_idx (int32)   2 rem_orig (int64, position in the original index)
 *   3 row_perm (int32, n: rows of chunk k in [chunk_ptr[k], chunk_ptr[k+1]), longest first)
 *   4 cb_off (int64, K+1: column blocks of chunk c)   5 colslot_vertex (int32, 64 per column block, -1 = padding)
 *   6 chunk_blk_off (int64, K+1: dense blocks whose rows are in chunk k)   7 blk_rb (int32, row block in its chunk)
 *   8 blk_cb (int32, column block)   9 blk_e0 (int64, n_blocks+1)   10 ent_pos (uint16, row_in_block << 8 | col_in_block)
 *   11 ent_orig (int64, position in the original index)   12 min_nnz_used (int32, K: threshold of every row chunk)
 * gnnstage_dense_plan_create_capped: the dense kernel serves the blocks of a row block in items of at most
 * item_blocks blocks, one workgroup per item and column half.  A launch (one row chunk) that fits one round of
 * workgroups takes as long as its longest item however many blocks it has, so every chunk takes the lowest rung of
 * a 5 % ladder from min_nnz (t -> max(t + 1, floor(1.05 t))) at which it has at most max_items items; a chunk that
 * does not get there below min_nnz_many (>= min_nnz) needs several rounds, every block costs time, and it takes
 * min_nnz_many.                                                                                              */
typedef struct gnnstage_dense_plan gnnstage_dense_plan;
int gnnstage_dense_plan_create(const int64_t *ptr, const int32_t *idx, int64_t n_vertices, int32_t n_chunks,
                               const int64_t *chunk_ptr, int32_t min_nnz, double min_share,
                               gnnstage_dense_plan **out);
int gnnstage_dense_plan_create_capped(const int64_t *ptr, const int32_t *idx, int64_t n_vertices, int32_t n_chunks,
                                      const int64_t *chunk_ptr, int32_t min_nnz, double min_share, int32_t item_blocks,
                                      int64_t max_items, int32_t min_nnz_many, gnnstage_dense_plan **out);
int64_t gnnstage_dense_plan_get(const gnnstage_dense_plan *plan, int32_t what, const void **data);
int gnnstage_dense_plan_destroy(gnnstage_dense_plan *plan);

/*
 * Per-kernel timing with HIP events on the launch stream.  kind: 0 forward aggregation,
 * 1 forward transform, 2 backward transposed aggregation, 3 input-gradient GEMM,
 * 4 weight-gradient GEMM (+bias gradient), 5 history copy, 6 other (masks, weight staging),
 * 7 long-row reduce of an aggregation.  gnnstage_profile_read synchronises the device, then
 * returns summed milliseconds and launch count of that kind for one layer (0 <= layer < L) or,
 * with layer < 0, over all layers.
 * gnnstage_profile_enable switches all kinds on or off; gnnstage_profile_select takes a bit mask of kinds
 * (bit k = kind k), for callers that want the events of a few kinds only inside a timed region (every
 * timed launch costs two event records on the stream).
 */
enum { GNNSTAGE_NKINDS = 8 };
int gnnstage_profile_enable(gnnstage_t *st, int32_t on);
int gnnstage_profile_select(gnnstage_t *st, uint32_t kind_mask);
int gnnstage_profile_read(gnnstage_t *st, int32_t kind, int32_t layer, double *ms, int64_t *launches);
int gnnstage_profile_reset(gnnstage_t *st);

/*
 * Diagnostic: what this GPU's memory system gives the access pattern of the aggregation (Algorithm 1's AGGREGATE
 * line reads one embedding row per neighbour), with no arithmetic and no index traffic around it.  Every 16-lane
 * group reads whole rows of row_bytes (a multiple of 256, at most 4096) at pseudo-random row numbers, eight rows in
 * flight per group, 2048 workgroups; a share hot_share of the draws goes to rows [0, hot_rows), the rest is uniform
 * over the n_rows rows of the table.  mode 0: plain loads, hot rows are the first rows of the table; 1: the same with
 * non-temporal loads; 2: plain loads, the hot rows spread evenly over the table (the case of a graph whose hubs
 * carry arbitrary ids); 3: non-temporal loads for the draws outside the hot rows only.  One warm-up launch, then n_launches timed with HIP events on hip_stream;
 * synchronises.  table: DEVICE, n_rows * row_bytes bytes, 16-byte aligned; sink: DEVICE, 4 bytes.
 * bytes_per_second (HOST) receives gathered bytes per second.  Returns 0, GNNSTAGE_EINVAL or GNNSTAGE_EHIP.
 */
int gnnstage_debug_gather_rate(const void *table, int64_t n_rows, int32_t row_bytes, int64_t gathers_per_launch,
                               int32_t n_launches, int64_t hot_rows, double hot_share, int32_t mode, uint32_t seed,
                               void *sink, void *hip_stream, double *bytes_per_second);

/* Diagnostic (host only, launches nothing): 1 when the dense-block launcher refuses a launch whose operand `missing` is
 * absent (0 zero row, 1 column slots, 2 selected source table, 3 partial tiles, 4 column scales / weight tiles,
 * 5 row scales; pattern_blocks != 0: blocks kept as bit patterns, else as weight tiles), 0 when it would launch,
 * -1 for an operand that the block kind does not have.  The kernel reads every operand without a test of its own. */
int gnnstage_debug_dense_rejects(int32_t missing, int32_t pattern_blocks);

/* Library version, e.g. 100 = 0.1.0 */
int gnnstage_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GNNSTAGE_H */
