// Shared declarations of the gnnstage HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16_t;

// Which chunks count as processed (Section 3.3, V_processed), one bit per chunk id.
// Passed by value as a kernel argument; supports up to 256 chunks.
struct ChunkMask {
  uint64_t w[4];
};
constexpr int kMaxChunks = 256;
constexpr int kMaxClasses = 32;  // source-id classes of the aggregation schedule (a 32-bit activity mask)
constexpr int kMaxSegs = 12;     // class segments one XCD may serve in a launch

// The word is picked with selects, not with an indexed access: a kernel that holds the mask as an argument
// would otherwise fetch the word from memory and wait for it (and for every other load in flight).
__host__ __device__ inline bool mask_test(const ChunkMask &m, uint32_t c) {
  const uint64_t lo = (c & 64u) ? m.w[1] : m.w[0], hi = (c & 64u) ? m.w[3] : m.w[2];
  return (((c & 128u) ? hi : lo) >> (c & 63u)) & 1ull;
}

// ---- aggregation (SpMM with current/history select) ---------------------------------
enum SpmmEpilogue : int {
  SPMM_PLAIN = 0,     // out = acc
  SPMM_MIX = 1,       // out = s_acc * acc + s_aux * aux[row]      (GCNII initial residual)
  SPMM_MASK = 2,      // out = aux[row] > 0 ? acc : 0              (ReLU derivative on the way back)
  SPMM_BIAS_RELU = 3, // out = max(acc + bias[c], 0)               (transform-first layers)
  SPMM_ADD = 4,       // out = acc + add[row - add_row0]           (GraphSage: the gradient through W_self joins)
  SPMM_ADD_MASK = 5   // out = aux[row] > 0 ? acc + add[row - add_row0] : 0
};
__host__ __device__ inline bool spmm_reads_aux(int e) { return e == SPMM_MIX || e == SPMM_MASK || e == SPMM_ADD_MASK; }
__host__ __device__ inline bool spmm_reads_add(int e) { return e == SPMM_ADD || e == SPMM_ADD_MASK; }

// Dropout behind an activation: threshold = ceil(rate * 2^24) (0: none), scale = 1 / (1 - rate), key = the
// layer's key of this pass, u0 = vertex id of the launch's first row.  Feature c of vertex u (rows of d features)
// survives when the top 24 bits of SplitMix64(key + (u * d + c + 1) * golden) reach the threshold.
struct LnDropout {
  uint32_t threshold;
  float scale;
  uint64_t key;
  int64_t u0;
};
__host__ __device__ inline uint64_t splitmix64_dev(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
__host__ __device__ inline bool dropout_keep(const LnDropout &dp, int64_t u, int d, int c) {
  const uint64_t r = splitmix64_dev(dp.key + (uint64_t)(u * d + c + 1) * 0x9E3779B97F4A7C15ull);
  return (uint32_t)(r >> 40) >= dp.threshold;
}

struct SpmmArgs {
  // sparse structure: packed index words (vertex | chunk << vbits) and weights
  const uint32_t *pidx;
  const float *val;
  // launch schedule
  const int32_t *task_row;
  const int64_t *task_e0;
  const int32_t *task_ne;
  const int32_t *task_slot;
  int64_t n_tasks;
  // The last n_short tasks are whole rows of at most a few entries (no partial slot).  The matrix-core kernel gives
  // them to extra workgroups of the same launch in which every 16-lane group owns a row of its own: a wave per
  // row would spend its life waiting for three dependent round trips to move a kilobyte or two.  The launcher
  // takes them off n_tasks; the vector-ALU kernel ignores the field and serves them like any other task.
  int64_t n_short;
  int64_t n_main_blocks;  // set by the launcher: workgroups from this index on serve the short rows
  // XCD-aware serving order.  Tasks [0, tail_task0) are pieces grouped by source-id class (class c at
  // cls_task0[c], cls_ntasks[c] of them).  Workgroups are dealt round-robin to the 8 XCDs; XCD x
  // (workgroups with index % 8 == x) serves up to kMaxSegs segments, segment s being the groups of four tasks
  // seg_g0[x][s] .. seg_g0[x][s] + seg_cnt[x][s] - 1 of class seg_cls[x][s].  Workgroups from
  // n_class_blocks on serve the tail.
  int32_t cls_task0[kMaxClasses], cls_ntasks[kMaxClasses];
  int32_t seg_cls[8][kMaxSegs], seg_g0[8][kMaxSegs], seg_cnt[8][kMaxSegs];
  int32_t n_class_blocks;
  int64_t tail_task0;
  const uint8_t *slot_class;  // class of every partial slot (255: none); pieces of inactive classes are not run
  uint32_t active_classes;
  int32_t all_classes_active;
  // long rows: pieces summed by the reduce kernel
  const int32_t *lr_row;
  const int32_t *lr_slot0;
  const int32_t *lr_nslots;
  int64_t n_long;
  float *partial;  // [n_slots][d] fp32
  // dense-block partial sums of a cut row: rows lr_dense0[i] + 128 * g (g < lr_ndense[i]) of dense_partial,
  // one per item of the row's row block; lr_item0[i] is the first of those items (for the activity test)
  const int32_t *lr_dense0;
  const int32_t *lr_ndense;
  const int32_t *lr_item0;
  const ChunkMask *item_chunks;
  const float *dense_partial;
  int32_t drop_unselected;  // the launch skips unselected entries: items without a chunk in the mask were not run
  // gathered operand: rows of width d, leading dimension src_ld
  const void *src_sel;    // read when the neighbour's chunk is in the mask
  const void *src_unsel;  // read otherwise; nullptr => the entry contributes zero
  int32_t d;
  int32_t src_ld;
  int32_t vbits;
  ChunkMask mask;
  // output rows: out[(row - out_row0) * out_ld + c], c < d; columns [d, out_ld) get zeros
  void *out;
  int32_t out_ld;
  int64_t out_row0;
  // epilogue
  int32_t epilogue;
  const void *aux;  // indexed by absolute row, leading dimension aux_ld, same dtype as src
  int32_t aux_ld;
  float s_acc, s_aux;
  const float *bias;  // SPMM_BIAS_RELU
  const void *add;    // SPMM_ADD / SPMM_ADD_MASK: rows indexed by row - add_row0, same dtype as src
  int32_t add_ld;
  int64_t add_row0;
  float mask_scale = 1.f;  // SPMM_MASK / SPMM_ADD_MASK: what passes the mask is scaled (1 / (1 - rate) of that dropout)
  // kernel choice (measurement and test switches, set by the stage from what it read at create)
  int32_t force_valu = 0;  // vector-ALU aggregation for bf16 rows too
  int32_t unroll = 2;      // gather slots per wave of the matrix-core aggregation: 2, 4 or 8
};

// which task the wave `wave` of workgroup `b` runs (-1: none)
__device__ inline int64_t spmm_task_index(const SpmmArgs &a, unsigned b, int wave) {
  if (b < (unsigned)a.n_class_blocks) {
    const int x = b & 7;
    int j = b >> 3;
#pragma unroll
    for (int s = 0; s < kMaxSegs; ++s) {
      const int cnt = a.seg_cnt[x][s];
      if (j < cnt) {
        const int cls = a.seg_cls[x][s];
        const int64_t t = ((int64_t)a.seg_g0[x][s] + j) * 4 + wave;
        return t < a.cls_ntasks[cls] ? a.cls_task0[cls] + t : -1;
      }
      j -= cnt;
    }
    return -1;
  }
  const int64_t t = a.tail_task0 + (int64_t)(b - a.n_class_blocks) * 4 + wave;
  return t < a.n_tasks ? t : -1;
}

// ---- dense blocks of an aggregation (bf16 rows of width 128 or 256) ---------------------------
// After ordering rows and columns by degree, the blocks that hold many entries are multiplied as dense
// 128 x 64 tiles on the matrix cores; the sparse kernels above only see the remaining entries.  An item
// is a run of blocks of one row block; it leaves a 128 x d fp32 tile of partial sums that the reduce
// kernel adds to the rows' sparse pieces.
constexpr int kDenseRB = 128, kDenseCB = 64;
constexpr int kDenseMaxItemBlocks = 32;  // blocks one workgroup multiplies before it writes its partial tile
struct DenseArgs {
  const int32_t *item_rb;         // row block (inside the chunk) of every item of this launch
  const int64_t *item_b0;         // its first block
  const int32_t *item_nb;         // and how many
  const ChunkMask *item_chunks;   // chunks its blocks' columns come from
  int32_t n_items;
  const int32_t *blk_cb;          // column block of every block: column slots 64 * cb ...
  const bf16_t *tiles;            // per block two 128 x 64 weight tiles (nearest bf16, then the remainder's bf16) as
                                  // launch_dense_expand writes them: [32-row group][16-column step][lane][8 values]
  // weights of the form s(row) * s(column) instead (bits != nullptr): per block 256 words of pattern bits
  // (word t: row t / 2, columns 32 * (t % 2) ..), s per column slot (0 = padding) and per row position of the chunk
  const uint32_t *bits;
  const float *colscale;
  const float *rowscale;          // [row blocks of the chunk * 128], zero past the chunk's last row
  const void *zero_row;           // at least 512 bytes of zeros, 16-byte aligned
  const uint32_t *colslot;        // vertex | chunk << vbits of every column slot, 0xffffffff = padding
  const void *src_sel;            // rows of vertices whose chunk is in the mask
  const void *src_unsel;          // rows of the others; nullptr => they contribute zero
  int32_t d, src_ld, vbits;
  ChunkMask mask;
  float *partial;                 // [n_items][128][d]
};
int launch_spmm_dense(const DenseArgs &a, hipStream_t s);
// Writes the weight tiles of n_blocks blocks (cleared by the caller) from their entry lists: entries
// [blk_e0[b], blk_e0[b + 1]) of block b, position = row << 8 | column (0xffff = padding), weight as two bf16
// halves (nearest bf16 in the low half of the word, the remainder's bf16 in the high half).
int launch_dense_expand(const int64_t *blk_e0, const uint16_t *ent_pos, const uint32_t *ent_w, void *tiles, int64_t n_blocks,
                        hipStream_t s);

enum DType : int { DT_F32 = 0, DT_BF16 = 1 };

// src dtype -> out dtype; returns hipError_t as int.  launch_spmm runs the per-task kernel,
// launch_spmm_reduce adds the pieces of long rows (needed whenever a.n_long > 0).
int launch_spmm(const SpmmArgs &a, int src_dtype, int out_dtype, hipStream_t s);
int launch_spmm_reduce(const SpmmArgs &a, int src_dtype, int out_dtype, hipStream_t s);

// ---- dense transforms -------------------------------------------------------------------
enum GemmEpilogue : int {
  EPI_FWD_GCN = 0,     // out = ReLU(acc + bias[n])
  EPI_FWD_GCNII = 1,   // out = ReLU((1-beta) aux[m][n] + beta acc)
  EPI_PLAIN = 2,       // out = acc
  EPI_DGRAD_GCNII = 3, // dp = (1-beta) aux[m][n] + beta acc; out = (1-alpha) dp; h0grad[m][n] += alpha dp
  EPI_MASK = 4,        // out = aux[m][n] > 0 ? acc : 0
  EPI_FWD_ADD = 5,     // out = ReLU(acc + bias[n] + aux[m][n])   (GraphSage: aux = h_v W_self)
  EPI_RES = 6          // out = acc + bias[n] + aux[m][n]         (ResGCN+: aux = h_v, no activation)
};

// C[M x N] = A[M x K] . Bt[N x Kp]^T.  Bt is an internal buffer: K-contiguous rows, zero padded to Kp,
// Kp % 8 == 0, compute dtype.  A is either such a padded buffer too, or any row-major matrix of fp32 or
// bf16 elements with K valid columns (read with bounds checks).
struct GemmNtArgs {
  const void *A;
  int32_t a_dtype;
  int32_t lda;
  const void *Bt;
  int32_t ldb;
  int32_t M, N, K, Kp;
  int32_t epilogue;
  const float *bias;
  const void *aux;
  int32_t aux_dtype;
  int32_t aux_ld;
  float alpha, beta;
  float *h0grad;  // fp32, pre-offset to the first row
  int32_t h0_ld;
  void *out;
  int32_t out_dtype;
  int32_t out_ld;
  int32_t out_pad;  // columns [N, out_pad) of every output row are written as zeros (0: none)
  int32_t vec_epi;  // set by the launcher: the epilogue may use 16-byte accesses
  float mask_scale = 1.f;  // EPI_MASK: what passes the mask is scaled (1 / (1 - rate) of that dropout)
  int32_t ws_min_rows = 65536;  // rows from which the weight-stationary kernel is used (tests force it on small inputs)
};
int launch_gemm_nt(const GemmNtArgs &a, int compute_dtype, hipStream_t s);

// dW[I x O] += scale * A[M x I]^T . B[M x O]   (reduction over the M rows of the chunk).
// B is an internal padded buffer in the compute dtype; A as for the NT product.
struct GemmTnArgs {
  const void *A;
  int32_t a_dtype;
  int32_t lda;
  const void *B;
  int32_t ldb;
  int32_t M, I, O;
  float scale;
  float *dW;       // fp32 [I][O]
  float *partial;  // fp32 scratch [splits][I][O]
  int32_t max_splits;
  float *dbias;         // optional (bf16 product only): dbias[o] += column sums of B, fused into the product
  float *bias_partial;  // fp32 scratch [splits][O]
  int32_t wide_min_rows = 65536;  // bf16 operands from this many rows on, with more than one 128 x 128 output tile: one
                                  // workgroup per row split computes the whole output (tests force it on small inputs)
};
int launch_gemm_tn(const GemmTnArgs &a, int compute_dtype, hipStream_t s);
// dst[o] += sum over the M rows of B[.][o]; partial: fp32 scratch [max_splits][O]
int launch_colsum_add(const void *B, int dtype, int ldb, int M, int O, float *partial, int max_splits, float *dst,
                      hipStream_t s);

// ---- LayerNorm + ReLU in front of the aggregation (ResGCN+ variant) -------------------------------
constexpr int kLnMaxWidth = 1024;  // a row lives in the registers of one wavefront
constexpr int kLnMaxWaves = 8192;  // wavefronts of one backward launch; the parameter-gradient scratch holds one
                                   // 2 x d block of sums per workgroup of four
// out[r][c] = Dropout(ReLU(gamma[c] * (x[r][c] - mean_r) / sqrt(var_r + eps) + beta[c])), c < d; zeros up to out_ld
int launch_ln_relu(const void *x, int x_dtype, int x_ld, const float *gamma, const float *beta, float eps, int64_t M, int d, void *out,
                   int out_dtype, int out_ld, const LnDropout &dp, hipStream_t s);
// Backward of the same for M rows: dr is the gradient of the activated rows.  out (may be NULL) receives the
// gradient of x plus, when res is not NULL, the rows of res (the residual branch); dgamma / dbeta get "+=" of
// the column sums in a fixed order (partial: fp32 scratch, kLnMaxWaves / 4 * 2 * d).
int launch_ln_relu_backward(const void *x, int x_dtype, int x_ld, const float *gamma, const float *beta, float eps, const void *dr,
                            int dr_dtype, int dr_ld, const void *res, int res_dtype, int res_ld, int64_t M, int d, void *out,
                            int out_dtype, int out_ld, float *partial, float *dgamma, float *dbeta, const LnDropout &dp,
                            hipStream_t s);
// dst[r][c] = src[r][c] for c < d, zero for d <= c < dst_ld
int launch_copy_rows(const void *src, int src_ld, void *dst, int dst_ld, int64_t M, int d, int dtype, hipStream_t s);

// ---- small kernels ------------------------------------------------------------------------
// Wt[N][Kp] (transposed) and Wn[K][Np] (plain) zero-padded copies of W[K][N] in the compute dtype
int launch_stage_weights(const void *W, int w_dtype, int K, int N, void *Wt, int Kp, void *Wn, int Np,
                         hipStream_t s);
// dY[m][c] = level[m][c] > 0 ? g[m][c] : 0 for c < d, zeros up to out_ld
// x[r][c] <- survives ? x[r][c] * scale : 0 in place, r < M, c < d (rows of leading dimension ld; dp.u0 = vertex of row 0)
int launch_dropout_rows(void *x, int dtype, int64_t M, int d, int ld, const LnDropout &dp, hipStream_t s);
// out = level > 0 ? g * scale : 0 (the ReLU derivative on the way back; scale = 1 / (1 - rate) of a dropout behind it)
int launch_relu_mask(const void *g, const void *level, int dtype, int64_t M, int d, void *out, int out_ld, float scale,
                     hipStream_t s);
int launch_copy(const void *src, void *dst, size_t bytes, hipStream_t s);
int launch_fill_zero(void *dst, size_t bytes, hipStream_t s);
// symmetric normalisation weights from row lengths: val[e] = 1/sqrt(len(row) * len(other))
int launch_gcn_norm(const int64_t *ptr, const uint32_t *pidx, int vbits, const int64_t *len_ptr, int64_t n,
                    float *val, hipStream_t s);

static inline int round_up(int x, int m) { return (x + m - 1) / m * m; }
