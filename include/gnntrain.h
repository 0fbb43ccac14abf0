/*
 * gnntrain — the epoch loop of Algorithm 1 around gnnstage handles, on one MI355X (gfx950).  C ABI.
 *
 * One epoch: draw the chunk order (Section 3.4, first technique: shuffled at the beginning of every
 * epoch); every chunk, in that order, goes through all stages (first to last) and the loss head; the
 * backward pass walks the chunks in the reverse order, last stage first; the weights are updated
 * (Algorithm 1, last line: the plain gradient step; Section 5 trains with Adam, learning rate 0.001);
 * the historical embeddings are refreshed after the epochs alpha, 2 alpha, ... (Section 3.4, second
 * technique: epoch t reads the embeddings of epoch alpha * floor((t - 1) / alpha)).
 *
 * The stages run back to back on this GPU: level L of stage s must be the same DEVICE buffer as level 0
 * of stage s + 1, and stage s + 1 must have been created with need_input_grad (its grad_in rows are the
 * upstream gradient of stage s).  On a pipeline of several GPUs each stage would sit on its own device
 * and this loop would be its schedule; here it is the sequential schedule, which computes the same values.
 *
 * The paper does not print its loss.  The head taken here is the usual one for node classification: a
 * linear classifier on the last level, logits = h W_o + b_o, and the mean softmax cross-entropy over the
 * labelled vertices.
 *
 * Ownership as in gnnstage.h: everything the descriptor points to stays with the caller, HOST arrays are
 * copied at create time, the library allocates no device memory (its state lives in the workspace).
 * Every function returns GNNSTAGE_OK or a negative GNNSTAGE_E* code.
 */
#ifndef GNNTRAIN_H
#define GNNTRAIN_H

#include "gnnstage.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gnntrain gnntrain_t; /* opaque, owned by the library */

enum { GNNTRAIN_SGD = 0, GNNTRAIN_ADAM = 1 };

/* One trainable tensor.  The optimiser works on the fp32 master copy; after every step it also writes the
 * copy the kernels read when that is a different buffer (bf16 stages: W[j] of gnnstage_desc, head_W). */
typedef struct {
  float *master;         /* DEVICE fp32, count elements; holds the initial value at create time */
  void *compute;         /* DEVICE, count elements of compute_dtype; NULL when the kernels read master */
  int32_t compute_dtype; /* GNNSTAGE_F32 or GNNSTAGE_BF16 */
  float *grad;           /* DEVICE fp32, count elements; zeroed by the loop at the start of every epoch */
  int64_t count;
} gnntrain_param;

typedef struct {
  int32_t n_stages;
  gnnstage_t *const *stages; /* HOST array, first to last; same graph size and chunks for all */
  /* loss head on level L of the last stage (n x d_top, that stage's dtype) */
  int32_t n_classes;
  const void *head_W;        /* DEVICE d_top x n_classes, dtype of the last stage */
  const float *head_b;       /* DEVICE fp32 n_classes */
  float *head_dW;            /* DEVICE fp32 d_top x n_classes, "+=" over the chunks */
  float *head_db;            /* DEVICE fp32 n_classes */
  const int32_t *labels;     /* DEVICE, one class id in [0, n_classes) per vertex */
  const uint8_t *train_mask; /* DEVICE, one byte per vertex (non-zero = labelled); NULL = all vertices */
  /* parameters of all stages and of the head, in the order they are stepped */
  int32_t n_params;
  const gnntrain_param *params; /* HOST array */
  int32_t optimizer;            /* GNNTRAIN_SGD: p -= lr (g + wd p);  GNNTRAIN_ADAM: Kingma & Ba, Algorithm 1 */
  float lr, beta1, beta2, eps, weight_decay;
  int32_t shuffle;    /* 0: chunks in index order every epoch */
  uint64_t seed;      /* of the chunk shuffling, and of the dropout decisions of stages that have dropout: stage s
                         gets gnnstage_set_dropout_seed(SplitMix64(seed + (epoch + 1) * 0x9E3779B97F4A7C15) + s) */
  int32_t alpha_hist; /* refresh period of the historical embeddings, >= 1 */
  int32_t history_swap; /* non-zero: refresh with gnnstage_update_history_swap (the level buffers of a stage trade places,
                           nothing but level 0 is copied) instead of update_history; the stages' level pointers then
                           come from gnnstage_level_buffers */
  void *workspace;    /* DEVICE, 256-byte aligned, >= gnntrain_workspace_size() bytes */
  size_t workspace_bytes;
} gnntrain_desc;

/* Device bytes the loop needs: optimiser moments, logits of one chunk, gradient of the logits for all
 * vertices, gradient rows of the last level for one chunk, per-vertex losses, staged head weights,
 * split-reduction scratch.  Host-only; 0 on an invalid descriptor. */
size_t gnntrain_workspace_size(const gnntrain_desc *desc);

/* Validates the descriptor against the stage handles (chaining of the level buffers, label range),
 * clears the optimiser state and synchronises.  *out is NULL on failure. */
int gnntrain_create(const gnntrain_desc *desc, gnntrain_t **out);

/* Runs epoch `epoch` (0-based; epochs must be run in order for the history schedule to mean what the
 * paper says, but the function itself only uses the number for the chunk order and the refresh test).
 * loss: HOST, receives the mean cross-entropy of this epoch's forward pass; with a non-NULL loss the call
 * synchronises the stream before returning, with NULL it is asynchronous. */
int gnntrain_epoch(gnntrain_t *tr, int64_t epoch, float *loss, void *hip_stream);

/* The chunk order the last epoch used (HOST, n_chunks entries). */
int gnntrain_last_order(const gnntrain_t *tr, int32_t *order);

int gnntrain_destroy(gnntrain_t *tr);
const char *gnntrain_last_error(const gnntrain_t *tr);

/* ---- the steps of the loop, exported one by one ------------------------------------------------- */

/* Section 3.4, first technique.  order: HOST, n_chunks entries.  Epoch e owns the SplitMix64 stream (Steele,
 * Lea, Flood 2014) that starts at state seed + (e + 1) * 0x9E3779B97F4A7C15; draw i is the generator's
 * output for state start + (i + 1) * 0x9E3779B97F4A7C15; a Fisher-Yates pass from the last position down
 * swaps position i with position draw mod (i + 1).  Host only. */
int gnntrain_chunk_order(uint64_t seed, int64_t epoch, int32_t n_chunks, int32_t shuffle, int32_t *order);

/* Softmax cross-entropy of `rows` vertices.  logits: DEVICE fp32 rows x ld (n_classes valid columns); bias
 * (DEVICE fp32, may be NULL) is added to them first.  For a labelled row: row_loss = log sum_c exp(z_c) -
 * z_label and dlogits_c = (softmax_c - [c = label]) * inv_n_train; an unlabelled row gets loss 0 and a zero
 * gradient.  dlogits: DEVICE rows x dl_ld of dl_dtype, columns [n_classes, dl_ld) are written as zeros.
 * labels / mask are indexed by row (pass pointers to the first row).  Asynchronous. */
int gnntrain_softmax_xent(const float *logits, int32_t ld, const float *bias, const int32_t *labels,
                          const uint8_t *mask, int64_t rows, int32_t n_classes, float inv_n_train, void *dlogits,
                          int32_t dl_dtype, int32_t dl_ld, float *row_loss, void *hip_stream);

/* out[0] = scale * sum of x[0 .. n), added in a fixed order (reproducible).  scratch: DEVICE, 1024 floats. */
int gnntrain_sum(const float *x, int64_t n, float scale, float *scratch, float *out, void *hip_stream);

/* gnntrain_sum for callers that cannot allocate or bring a scratch buffer: code under HIP graph capture, tight
 * serving loops, harnesses that forbid allocation.  Same kernels, same order of additions, same result bit for
 * bit; the 1024 block sums go to an array that lives inside the library's device image (4 KB on every GPU the
 * library runs on, held until the process ends).  Calls no allocating routine.  Its address on the current device
 * is looked up at the first call on that device.  n may be at most GNNTRAIN_SUM_STATIC_MAX_N, beyond that the
 * call returns GNNSTAGE_ENOTSUP (gnntrain_last_error(NULL) says why; also for EINVAL and EHIP).  Nothing in the
 * array has to be cleared between calls (the first launch writes every slot the second reads), but every call on
 * one GPU uses the same array: calls that overlap in time on one GPU (two streams) race.  x, out: DEVICE. */
#define GNNTRAIN_SUM_STATIC_MAX_N 2147483647LL
int gnntrain_sum_static(const float *x, int64_t n, float scale, float *out, void *hip_stream);

/* One optimiser step on one tensor (t = 1, 2, ... for Adam's bias correction).  compute may be NULL. */
int gnntrain_adam_step(float *p, const float *g, float *m, float *v, void *compute, int32_t compute_dtype,
                       int64_t count, float lr, float beta1, float beta2, float eps, float weight_decay, int64_t t,
                       void *hip_stream);
int gnntrain_sgd_step(float *p, const float *g, void *compute, int32_t compute_dtype, int64_t count, float lr,
                      float weight_decay, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* GNNTRAIN_H */
