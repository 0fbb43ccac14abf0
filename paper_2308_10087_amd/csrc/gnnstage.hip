// C-ABI entry points of the stage library: descriptor validation, workspace layout, host
// planning at create time, and the per-chunk launch sequences (Algorithm 1's inner loops and
// the matching backward pass).  All device work is issued on the caller's stream.
#include <stdio.h>
#include "guard.h"
#include <memory>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <string>
#include <utility>
#include <vector>

#include "../../include/gnnstage.h"
#include "common.h"
#include "plan.h"

namespace {

// Row splits of a weight-gradient product (fp32 partial outputs, added in a fixed order).  512 = two workgroups per CU in
// one round: measured on the 2.45 M x 128 x 128 products of the 8-layer configuration, 256 / 384 / 512 / 640 / 768 /
// 1024 splits take 3.08 / 2.62 / 2.56 / 3.24 / 3.01 / 2.91 ms per step.
constexpr int kMaxSplits = 512;
constexpr size_t kAlign = 256;

std::string g_create_error;

// Measurement and test switches.  Defaults are the product path.  The environment is read ONCE per
// gnnstage_workspace_size / gnnstage_create call (both must see the same values) and the result is kept in
// the handle; nothing on the launch path looks at the environment.
//   GNNSTAGE_SPLIT_EDGES (>= 64)      fixed length of the pieces long rows are cut into
//   GNNSTAGE_XCD_CLASSES (1..32)      source-id classes (1 = off)
//   GNNSTAGE_CLASS_MIN_ROW            rows from this length on are cut by class
//   GNNSTAGE_DENSE=0                  no dense blocks
//   GNNSTAGE_DENSE_MIN_NNZ            entries a 128 x 64 block needs to be multiplied as a dense block
//   GNNSTAGE_DENSE_MIN_SHARE          share of all entries that must fall into such blocks
//   GNNSTAGE_DENSE_MIN_ENTRIES        dense entries per chunk below which the plan stays off
//   GNNSTAGE_ORDER=aggregate|transform  one layer order for every GCN layer
//   GNNSTAGE_SPMM_VALU                vector-ALU aggregation for bf16 rows too
//   GNNSTAGE_SPMM_UNROLL (2, 4, 8)    gather slots per wave of the matrix-core aggregation
//   GNNSTAGE_GEMM_WS_MIN_ROWS         rows from which the weight-stationary product is used
//   GNNSTAGE_GEMM_WIDE_MIN_ROWS       rows from which a weight-gradient product of up to 256 x 256 outputs is one workgroup per split
//   GNNSTAGE_WGRAD_DEFER=0            weight gradients per chunk instead of one product per layer at the end of the pass
//   GNNSTAGE_HOT_CLASSES (0 = off, 2..32: on whatever the table size)   classes of the hottest sources
//   GNNSTAGE_HOT_ROWS                 sources per such class
//   GNNSTAGE_HOT_MIN_ROW              rows from this length on are cut by hotness class
//   GNNSTAGE_SHORT_ROW (0 = off)      whole rows of at most this many entries are served a row per 16-lane group
struct Tuning {
  int split_edges = 0;          // 0: from the launch size
  int xcd_classes = 0;          // 0: from the size of the gathered table
  int class_min_row = 128;      // measured: shorter rows than this cost more in partial sums than their locality gains
  bool dense = true;
  int dense_min_nnz = 0;        // 0: the defaults below
  double dense_min_share = 0.2;
  double dense_min_entries = 2e6;
  int order = 0;                // 0 auto, 1 aggregate first, 2 transform first
  bool spmm_valu = false;
  int spmm_unroll = 2;          // two slots leave room for eight waves per SIMD, which measured best on every workload
  int gemm_ws_min_rows = 65536;
  int gemm_wide_min_rows = 65536;  // weight-gradient products from this many rows on read each operand once (one workgroup per split)
  bool wgrad_defer = true;
  int hot_classes = -1;         // -1: 16 for gathered tables beyond 256 MB, none below
  int hot_rows = 0;             // 0: as many rows as fit an XCD's 4 MB L2
  int hot_min_row = 2048;       // measured on the 10 M vertex graph: 512 -> 142.8, 1024 -> 140.6, 2048 -> 140.4 ms per step (off: 143.2)
  int short_row = -1;           // whole rows of at most this many entries are served a row per 16-lane group (0: none;
                                // -1: 4 for gathered tables beyond 256 MB, none below: 141.2 against 143.2 ms per step there,
                                // nothing or a small loss on tables that sit in a cache)
};

Tuning read_tuning() {
  Tuning t;
  const char *e;
  if ((e = getenv("GNNSTAGE_SPLIT_EDGES")) && atoi(e) >= 64) t.split_edges = atoi(e);
  if ((e = getenv("GNNSTAGE_XCD_CLASSES")) && atoi(e) >= 1 && atoi(e) <= kMaxClasses) t.xcd_classes = atoi(e);
  if ((e = getenv("GNNSTAGE_CLASS_MIN_ROW")) && atoi(e) >= 1) t.class_min_row = atoi(e);
  if ((e = getenv("GNNSTAGE_DENSE")) && atoi(e) == 0) t.dense = false;
  if ((e = getenv("GNNSTAGE_DENSE_MIN_NNZ")) && atoi(e) >= 1) t.dense_min_nnz = atoi(e);
  if ((e = getenv("GNNSTAGE_DENSE_MIN_SHARE"))) t.dense_min_share = atof(e);
  if ((e = getenv("GNNSTAGE_DENSE_MIN_ENTRIES"))) t.dense_min_entries = atof(e);
  if ((e = getenv("GNNSTAGE_ORDER"))) t.order = !strcmp(e, "aggregate") ? 1 : !strcmp(e, "transform") ? 2 : 0;
  if (getenv("GNNSTAGE_SPMM_VALU")) t.spmm_valu = true;
  if ((e = getenv("GNNSTAGE_SPMM_UNROLL"))) t.spmm_unroll = atoi(e);
  if ((e = getenv("GNNSTAGE_GEMM_WS_MIN_ROWS"))) t.gemm_ws_min_rows = atoi(e);
  if ((e = getenv("GNNSTAGE_GEMM_WIDE_MIN_ROWS"))) t.gemm_wide_min_rows = atoi(e);
  if ((e = getenv("GNNSTAGE_WGRAD_DEFER")) && atoi(e) == 0) t.wgrad_defer = false;
  if ((e = getenv("GNNSTAGE_HOT_CLASSES")) && atoi(e) >= 0 && atoi(e) <= kMaxClasses) t.hot_classes = atoi(e);
  if ((e = getenv("GNNSTAGE_HOT_ROWS")) && atoi(e) >= 1) t.hot_rows = atoi(e);
  if ((e = getenv("GNNSTAGE_HOT_MIN_ROW")) && atoi(e) >= 1) t.hot_min_row = atoi(e);
  if ((e = getenv("GNNSTAGE_SHORT_ROW")) && atoi(e) >= 0) t.short_row = atoi(e);
  return t;
}

// Longest piece of a row that one wavefront handles in an aggregation over `entries` entries.  A wave
// streams roughly 16 entries per microsecond, so the longest task bounds the tail of the launch: pieces
// shrink with the launch (about 16k pieces' worth of work per launch), within [256, 4096].
int split_edges_for(const Tuning &t, int64_t entries) {
  if (t.split_edges >= 64) return t.split_edges;
  int64_t s = (entries / 16384 + 63) / 64 * 64;
  if (s < 256) s = 256;
  if (s > 4096) s = 4096;
  return (int)s;
}

// Source-id classes (one per XCD) pay when one class's slice of the gathered table has a chance to
// live in an XCD's L2 and the memory-side cache; for tables far beyond that they only add partial sums.
int xcd_classes_setting(const Tuning &t, int64_t table_bytes) {
  if (t.xcd_classes >= 1) return t.xcd_classes;
  return table_bytes <= (int64_t)256 << 20 ? 8 : 1;
}

// Hotness classes, for tables that fit no cache.  On a power-law graph a small set of sources takes a large share
// of all gathers (10 M vertices, 21 entries per row: the 130 k most frequent sources are 45 % of the entries), but
// between two uses of such a row an XCD streams far more than its 4 MB L2 holds.  So the hottest sources are cut
// into classes of as many rows as fit one L2, long rows get their entries ordered by hotness and are cut at the
// class bounds, and the pieces of a class run together on one XCD (the class machinery above): a hot row is
// fetched once per launch and XCD instead of once per use.  The rest of every row, and all short rows, gather
// as before.  Off when id-range classes are forced (GNNSTAGE_XCD_CLASSES).
int hot_classes_setting(const Tuning &t, int64_t table_bytes) {
  if (t.xcd_classes >= 1) return 0;
  if (t.hot_classes >= 0) return t.hot_classes >= 2 ? t.hot_classes : 0;
  return table_bytes > (int64_t)256 << 20 ? 16 : 0;
}
int64_t hot_rows_setting(const Tuning &t, int64_t row_bytes) {
  if (t.hot_rows >= 1) return t.hot_rows;
  return std::max<int64_t>(64, ((int64_t)4 << 20) / std::max<int64_t>(row_bytes, 1));
}

// Lower bounds of the source-id classes: equal id ranges, except that a bound moves onto a chunk boundary
// that lies within a quarter of a class width of it.  Chunks that line up with classes (equal chunks, a
// multiple of the class count) then never straddle two classes, and a backward launch touches exactly the
// classes of its processed chunks.
std::vector<int64_t> class_bounds(int64_t n, int classes, const std::vector<int64_t> &chunk_ptr) {
  std::vector<int64_t> lo((size_t)classes + 1);
  for (int q = 0; q <= classes; ++q) lo[(size_t)q] = ((int64_t)q * n + classes - 1) / classes;
  const int64_t tol = n / (4 * (int64_t)classes);
  for (int q = 1; q < classes; ++q) {
    int64_t best = -1;
    for (const int64_t cb : chunk_ptr)
      if (std::llabs(cb - lo[(size_t)q]) <= tol && (best < 0 || std::llabs(cb - lo[(size_t)q]) < std::llabs(best - lo[(size_t)q])))
        best = cb;
    if (best > 0 && best < n) lo[(size_t)q] = best;
  }
  return lo;
}

// Class bounds for the rows [r0, r1) of an index (one chunk's launch): equal shares of those rows' ENTRIES rather than
// of the id range, so that a chunk whose neighbours cluster in a few id ranges (chunks from a locality-aware
// partitioner: about half of a chunk's neighbours are its own vertices) still spreads over all classes, its heavy
// range cut into slices that fit an L2.  A bound moves to a chunk boundary that lies within a quarter of a class share
// (in entries): classes made of whole chunks are skipped as a whole by launches that drop those chunks.  On a
// uniformly numbered graph this gives the equal, chunk-aligned id ranges of class_bounds.
std::vector<int64_t> class_bounds_by_entries(const int64_t *ptr, const int32_t *idx, int64_t n, int64_t r0, int64_t r1, int classes,
                                             const std::vector<int64_t> &chunk_ptr) {
  if (classes <= 1 || idx == nullptr || ptr[r1] == ptr[r0]) return class_bounds(n, classes, chunk_ptr);
  std::vector<int64_t> mass((size_t)n + 1, 0);  // mass[u + 1] = entries of these rows whose source is u, then prefix sums
  for (int64_t e = ptr[r0]; e < ptr[r1]; ++e) mass[(size_t)idx[e] + 1] += 1;
  for (int64_t u = 0; u < n; ++u) mass[(size_t)u + 1] += mass[(size_t)u];
  const int64_t total = mass[(size_t)n];
  const int64_t tol = total / (4 * (int64_t)classes);
  std::vector<int64_t> lo((size_t)classes + 1, 0);
  lo[(size_t)classes] = n;
  for (int q = 1; q < classes; ++q) {
    const int64_t target = total / classes * q + total % classes * q / classes;
    int64_t b = std::lower_bound(mass.begin(), mass.end(), target) - mass.begin();
    int64_t best = -1;
    for (const int64_t cb : chunk_ptr) {
      const int64_t dist = std::llabs(mass[(size_t)cb] - target);
      if (cb > 0 && cb < n && dist <= tol && (best < 0 || dist < std::llabs(mass[(size_t)best] - target))) best = cb;
    }
    if (best >= 0) b = best;
    lo[(size_t)q] = std::min<int64_t>(std::max<int64_t>(b, lo[(size_t)q - 1]), n);
  }
  return lo;
}

// Dense blocks: switched on for bf16 stages whose aggregations all gather rows of width 128 or 256.
// Threshold: entries a 128 x 64 block needs; default: from 3.4 % of its cells upwards, as low as the chunk's launch
// still fits one round of workgroups, 5 % for a chunk that needs several (see dense_max_items); the same for blocks
// kept as weight tiles, whose curve is flat from 278 to 500: 18.7 - 18.9 ms per c1 step with the caller's weights.
int dense_min_nnz(const Tuning &t) { return t.dense_min_nnz >= 1 ? t.dense_min_nnz : kDenseRB * kDenseCB * 34 / 1000; }
// for a chunk whose launch needs several rounds of workgroups: every block costs time there
int dense_min_nnz_many(const Tuning &t) { return t.dense_min_nnz >= 1 ? t.dense_min_nnz : kDenseRB * kDenseCB / 20; }
// Items (runs of at most 32 blocks of one row block) of a launch that fits one round of workgroups: one workgroup
// per item and 128-column half, two workgroups per CU, 256 CUs; a tenth more is harmless because short items end
// early.  Such a launch takes as long as its longest item, so blocks down to the low threshold are free; beyond it
// the extra workgroups wait for a second round.
int64_t dense_max_items(int widest) { return (int64_t)(2 * 256 * 11 / 10) / std::max(1, widest / 128); }
// A dense launch has a fixed cost (its longest item runs 32 blocks one after the other, some tens of
// microseconds); it only pays when it takes a lot of entries off the sparse kernel: at least
// Tuning::dense_min_entries per chunk on average (the sparse kernel gathers about 40 entries per nanosecond).
constexpr int kDenseItemBlocks = kDenseMaxItemBlocks;

struct TaskList {
  int64_t n_tasks = 0, n_long = 0, n_slots = 0;
  int64_t n_short = 0;  // the last n_short tasks are whole rows of at most Tuning::short_row entries
  int32_t *task_row = nullptr;
  int64_t *task_e0 = nullptr;
  int32_t *task_ne = nullptr;
  int32_t *task_slot = nullptr;
  int32_t *lr_row = nullptr, *lr_slot0 = nullptr, *lr_nslots = nullptr;
  // class sections of the task list (class c = tasks [cls_off[c], cls_off[c+1]); tail from cls_off[8])
  int n_classes = 0;                      // 0: no class sections
  int64_t cls_off[kMaxClasses + 1] = {};  // tail starts at cls_off[n_classes]
  uint8_t *slot_class = nullptr;
  // entries of every class section by the chunk of the gathered vertex ([class * K + chunk]): what a launch
  // that drops unselected entries really gathers from each class
  std::vector<int64_t> cls_chunk_entries;
  // dense-block parts of the cut rows and the items of this chunk (dense plan active only)
  int32_t *lr_dense0 = nullptr, *lr_ndense = nullptr, *lr_item0 = nullptr;
  int64_t item0 = 0;  // first item of the chunk in the direction's item arrays
  int n_items = 0;
};

// Sizes that depend only on row lengths: number of tasks / long rows / slots of every chunk.
struct PlanCounts {
  std::vector<int64_t> tasks, longs, slots;
  std::vector<int> split;
  int64_t total_slots = 0;
  int64_t total_tasks = 0, total_longs = 0, max_slots = 0;
};

// Upper bounds (from row lengths alone) on tasks / cut rows / slots of every chunk: a row cut by
// source class adds at most one extra piece per class.
PlanCounts count_plan(const Tuning &tune, const int64_t *ptr, const std::vector<int64_t> &chunk_ptr, int classes, int min_row,
                      const uint8_t *force = nullptr) {
  PlanCounts pc;
  const int K = (int)chunk_ptr.size() - 1;
  pc.tasks.assign(K, 0);
  pc.longs.assign(K, 0);
  pc.slots.assign(K, 0);
  pc.split.assign(K, 0);
  for (int c = 0; c < K; ++c) {
    const int split = split_edges_for(tune, ptr[chunk_ptr[c + 1]] - ptr[chunk_ptr[c]]);
    pc.split[c] = split;
    for (int64_t r = chunk_ptr[c]; r < chunk_ptr[c + 1]; ++r) {
      const int64_t len = ptr[r + 1] - ptr[r];
      const bool by_src = classes > 1 && len >= min_row;
      if (by_src || len > split || (force && force[r])) {
        const int64_t pieces = (len + split - 1) / split + (by_src ? classes + 1 : 0);  // + 1: the run beyond the classes
        pc.tasks[c] += pieces;
        pc.slots[c] += pieces;
        pc.longs[c] += 1;
      } else {
        pc.tasks[c] += 1;
      }
    }
    pc.total_tasks += pc.tasks[c];
    pc.total_longs += pc.longs[c];
    pc.total_slots += pc.slots[c];
    if (pc.slots[c] > pc.max_slots) pc.max_slots = pc.slots[c];
  }
  return pc;
}

// Everything the host plans for one aggregation direction before anything is uploaded.
struct HostDir {
  DensePlan dp;
  const int64_t *ptr = nullptr;   // the index the sparse kernels see: the original one, or the dense plan's remainder
  const int32_t *idx = nullptr;
  int64_t nnz = 0;
  std::vector<uint8_t> force;     // rows with dense parts (they always write partial sums)
  HotOrder hot;                   // active: idx is hot.idx (long rows ordered by hotness), hot.rank the ranks in that order
  int min_row = 128;              // rows from this length on are cut by class
  PlanCounts pc;
  std::vector<int32_t> item_rb, item_nb;
  std::vector<int64_t> item_b0;
  std::vector<ChunkMask> item_chunks;
  std::vector<int64_t> chunk_item_off;  // K + 1
  std::vector<int64_t> rowscale_off;    // K + 1: chunk k owns 128 scale slots per row block
  int64_t max_items = 0;
  bool dense() const { return dp.active; }
  int64_t padded_entries() const {  // entry lists padded to multiples of eight (16-byte loads)
    int64_t t = 0;
    for (int64_t b = 0; b < dp.n_blocks(); ++b) t += (dp.blk_e0[(size_t)b + 1] - dp.blk_e0[(size_t)b] + 7) / 8 * 8;
    return t;
  }
  const uint8_t *force_ptr() const { return dp.active ? force.data() : nullptr; }
};

void host_mask_set(ChunkMask &m, int c) { m.w[c >> 6] |= 1ull << (c & 63); }

bool make_host_dir(const Tuning &tune, const int64_t *ptr, const int32_t *idx, int64_t n, const std::vector<int64_t> &chunk_ptr,
                   int classes, bool hot, bool want_orig, bool try_dense, int dense_width, HostDir &h) {
  const int K = (int)chunk_ptr.size() - 1;
  h.ptr = ptr;
  h.idx = idx;
  h.nnz = ptr[n];
  h.chunk_item_off.assign((size_t)K + 1, 0);
  h.rowscale_off.assign((size_t)K + 1, 0);
  for (int k = 0; k < K; ++k)
    h.rowscale_off[(size_t)k + 1] = h.rowscale_off[(size_t)k] + (chunk_ptr[(size_t)k + 1] - chunk_ptr[(size_t)k] + kDenseRB - 1) / kDenseRB * kDenseRB;
  if (try_dense) {
    // share of all entries that must be dense: the relative threshold, or the absolute one if that asks for more
    const double nnz = (double)ptr[n];
    const double share = std::max(tune.dense_min_share, nnz > 0 ? tune.dense_min_entries * K / nnz : 0.0);
    if (!build_dense_plan(ptr, idx, n, K, chunk_ptr.data(), dense_min_nnz(tune), share, h.dp, kDenseItemBlocks, dense_max_items(dense_width),
                          dense_min_nnz_many(tune)))
      return false;
  }
  if (h.dp.active) {
    const DensePlan &dp = h.dp;
    h.ptr = dp.rem_ptr.data();
    h.idx = dp.rem_idx.data();
    h.nnz = (int64_t)dp.rem_idx.size();
    h.force.assign((size_t)n, 0);
    std::vector<int> chunk_of_cb((size_t)dp.cb_off[(size_t)K]);
    for (int c = 0; c < K; ++c)
      for (int64_t b = dp.cb_off[(size_t)c]; b < dp.cb_off[(size_t)c + 1]; ++b) chunk_of_cb[(size_t)b] = c;
    for (int k = 0; k < K; ++k) {
      int64_t b = dp.chunk_blk_off[(size_t)k];
      const int64_t b_end = dp.chunk_blk_off[(size_t)k + 1];
      while (b < b_end) {  // runs of blocks of one row block, at most kDenseItemBlocks each
        int64_t e = b;
        ChunkMask m{};
        while (e < b_end && dp.blk_rb[(size_t)e] == dp.blk_rb[(size_t)b] && e - b < kDenseItemBlocks) {
          host_mask_set(m, chunk_of_cb[(size_t)dp.blk_cb[(size_t)e]]);
          ++e;
        }
        h.item_rb.push_back(dp.blk_rb[(size_t)b]);
        h.item_b0.push_back(b);
        h.item_nb.push_back((int32_t)(e - b));
        h.item_chunks.push_back(m);
        const int64_t r0 = chunk_ptr[(size_t)k] + (int64_t)dp.blk_rb[(size_t)b] * kDenseRB;
        for (int64_t r = r0; r < std::min<int64_t>(r0 + kDenseRB, chunk_ptr[(size_t)k + 1]); ++r)
          h.force[(size_t)dp.row_perm[(size_t)r]] = 1;
        b = e;
      }
      h.chunk_item_off[(size_t)k + 1] = (int64_t)h.item_rb.size();
      h.max_items = std::max(h.max_items, h.chunk_item_off[(size_t)k + 1] - h.chunk_item_off[(size_t)k]);
    }
  }
  h.min_row = hot ? tune.hot_min_row : tune.class_min_row;
  if (hot && classes > 1) {  // on the index the sparse kernels see (the dense plan's remainder, if there is one)
    if (!build_hot_order(h.ptr, h.idx, n, h.min_row, want_orig, h.hot)) return false;
    h.idx = h.hot.idx.data();
  }
  h.pc = count_plan(tune, h.ptr, chunk_ptr, classes, h.min_row, h.force_ptr());
  return true;
}

struct Bump {
  size_t off = 0;
  size_t take(size_t bytes) {
    const size_t at = off;
    off += (bytes + kAlign - 1) / kAlign * kAlign;
    return at;
  }
};

struct Layout {
  size_t row_ptr, pcol, val, t_ptr, prow, tval;
  size_t f_task_row, f_task_e0, f_task_ne, f_task_slot, f_lr_row, f_lr_slot0, f_lr_n;
  size_t b_task_row, b_task_e0, b_task_ne, b_task_slot, b_lr_row, b_lr_slot0, b_lr_n;
  size_t f_slot_class, b_slot_class;
  size_t rem_ptr[2];  // row pointers of the remainder index per direction (dense plan active), else unused
  // dense plan per direction (0 forward, 1 transposed)
  size_t d_blk_cb[2], d_blk_e0[2], d_ent_pos[2], d_ent_w[2], d_colslot[2], d_tiles[2];
  size_t d_bits[2], d_colscale[2], d_rowscale[2];  // weights of the form s(row) * s(column): patterns and scales
  size_t d_item_rb[2], d_item_b0[2], d_item_nb[2], d_item_chunks[2];
  size_t d_lr_dense0[2], d_lr_ndense[2], d_lr_item0[2];
  size_t dense_partial, zero_row;
  size_t partial;
  std::vector<size_t> Z, dZ, Wt, Wn, Tc, Th;
  std::vector<size_t> dY;  // deferred weight gradients: dL/d(pre-activation) of every aggregate-first layer, all n rows
  std::vector<size_t> Wt_self, Wn_self;  // GraphSage: staged copies of W_self (Wt / Wn then hold W_neigh)
  size_t self_fwd = 0, self_bwd = 0;      // GraphSage: h_v W_self of a chunk (fp32), dY W_self^T of a chunk
  size_t res_dr = 0, ln_partial = 0;      // ResGCN+: gradient of the activated rows of a chunk; parameter-gradient scratch
  size_t G[2];
  size_t gemm_partial, bias_partial;
  size_t total;
};

struct Shape {
  int64_t n = 0, nnz = 0;
  int K = 0, L = 0;
  std::vector<int64_t> chunk_ptr;
  std::vector<int> dims, ld;
  std::vector<char> tf;  // per layer: 1 = transform first (gather rows of width d_{j+1}), 0 = aggregate first
  int dtype = 0, level0_f32 = 0, variant = 0, need_input_grad = 0;
  Tuning tune;
  bool has_bias() const { return variant != GNNSTAGE_GCNII; }
  // One weight-gradient product per layer over all rows at the end of the backward pass instead of one per chunk
  // (the rows of dL/d(pre-activation) are kept for the whole pass): a per-chunk product of a few ten thousand rows
  // runs at its launch and latency floor.  Not for ResGCN+ stages (their backward is a path of its own).
  bool defer_wgrad() const { return tune.wgrad_defer && variant != GNNSTAGE_RESGCN; }
  bool sage() const { return variant == GNNSTAGE_SAGE; }
  bool res() const { return variant == GNNSTAGE_RESGCN; }
  // elements of one weight matrix: GraphSage stacks [W_self ; W_neigh]
  size_t w_half(int j) const { return (size_t)dims[j] * dims[j + 1]; }
  int elt() const { return dtype == GNNSTAGE_BF16 ? 2 : 4; }
  int level_elt(int j) const { return (j == 0 && level0_f32) ? 4 : elt(); }
  // source classes for the aggregation schedule, decided by the widest bf16/fp32 table that is gathered
  int64_t widest_row_bytes() const {  // of the widest row any aggregation of the stage gathers
    int64_t widest = 0;
    for (int j = 0; j < L; ++j)
      widest = std::max<int64_t>(widest, tf[j] ? (int64_t)dims[j + 1] * elt()
                                               : std::max<int64_t>((int64_t)dims[j] * level_elt(j), (int64_t)dims[j] * elt()));
    return widest;
  }
  // classes of the hottest sources instead of id-range classes (tables that fit no cache)
  bool hot() const { return hot_classes_setting(tune, n * widest_row_bytes()) >= 2; }
  int64_t hot_rows() const { return hot_rows_setting(tune, widest_row_bytes()); }
  int short_row() const { return tune.short_row >= 0 ? tune.short_row : (n * widest_row_bytes() > ((int64_t)256 << 20) ? 4 : 0); }
  int classes() const {
    if (hot()) return hot_classes_setting(tune, n * widest_row_bytes());
    return xcd_classes_setting(tune, n * widest_row_bytes());
  }
  // dense blocks serve the matrix-core aggregation only: every aggregation of the stage must gather bf16 rows
  // of width 128 or 256
  int dense_width() const {  // the widest rows the dense kernel gathers (one workgroup per 128 columns)
    int wdt = 128;
    for (int j = 0; j < L; ++j) wdt = std::max(wdt, tf[j] ? dims[j + 1] : dims[j]);
    return wdt;
  }
  bool dense_ok() const {
    if (dtype != GNNSTAGE_BF16 || !tune.dense) return false;
    for (int j = 0; j < L; ++j) {
      const int wdt = tf[j] ? dims[j + 1] : dims[j];
      if (wdt != 128 && wdt != 256) return false;
      if (!tf[j] && j == 0 && level0_f32) return false;
    }
    return true;
  }
  int64_t max_rows() const {
    int64_t m = 0;
    for (int c = 0; c < K; ++c) m = std::max<int64_t>(m, chunk_ptr[c + 1] - chunk_ptr[c]);
    return m;
  }
};

bool read_shape(const gnnstage_desc *d, Shape &s, std::string &err) {
  if (!d) { err = "descriptor is NULL"; return false; }
  if (d->n_vertices <= 0 || d->nnz < 0) { err = "n_vertices must be positive and nnz non-negative"; return false; }
  if (!d->row_ptr || !d->chunk_ptr || !d->dims) { err = "row_ptr, chunk_ptr and dims must not be NULL"; return false; }
  if (d->n_chunks <= 0 || d->n_chunks > kMaxChunks) { err = "n_chunks must be in [1, 256]"; return false; }
  if (d->n_layers <= 0 || d->n_layers > 1024) { err = "n_layers must be in [1, 1024]"; return false; }
  if (d->dtype != GNNSTAGE_F32 && d->dtype != GNNSTAGE_BF16) { err = "unknown dtype"; return false; }
  if (d->variant != GNNSTAGE_GCN && d->variant != GNNSTAGE_GCNII && d->variant != GNNSTAGE_SAGE &&
      d->variant != GNNSTAGE_RESGCN) {
    err = "unknown variant";
    return false;
  }
  s.n = d->n_vertices;
  s.nnz = d->nnz;
  s.K = d->n_chunks;
  s.L = d->n_layers;
  s.dtype = d->dtype;
  s.level0_f32 = (d->dtype == GNNSTAGE_BF16 && d->level0_f32) ? 1 : 0;
  s.variant = d->variant;
  s.need_input_grad = d->need_input_grad ? 1 : 0;
  s.chunk_ptr.assign(d->chunk_ptr, d->chunk_ptr + s.K + 1);
  if (s.chunk_ptr[0] != 0 || s.chunk_ptr[s.K] != s.n) { err = "chunk_ptr must start at 0 and end at n_vertices"; return false; }
  for (int c = 0; c < s.K; ++c)
    if (s.chunk_ptr[c] > s.chunk_ptr[c + 1]) { err = "chunk_ptr must be non-decreasing"; return false; }
  s.dims.assign(d->dims, d->dims + s.L + 1);
  s.ld.resize(s.L + 1);
  for (int j = 0; j <= s.L; ++j) {
    if (s.dims[j] <= 0 || s.dims[j] > (1 << 20)) { err = "every level width must be in [1, 2^20]"; return false; }
    if (s.dtype == GNNSTAGE_BF16 && (s.dims[j] & 1) && !(j == 0 && s.level0_f32)) {
      err = "bf16 levels need an even width";
      return false;
    }
    s.ld[j] = round_up(s.dims[j], 8);
  }
  if (s.variant == GNNSTAGE_GCNII || s.res()) {
    for (int j = 1; j <= s.L; ++j)
      if (s.dims[j] != s.dims[0]) { err = "GCNII and ResGCN+ need equal widths at every level"; return false; }
    if (s.level0_f32) { err = "GCNII and ResGCN+ do not take an fp32 level 0"; return false; }
    if (s.res() && s.dims[0] > kLnMaxWidth) { err = "ResGCN+ rows are limited to 1024 columns"; return false; }
  }
  // Layer order.  (A_hat H) W == A_hat (H W) and the select is per edge, so a GCN layer may apply W
  // before the aggregation; that pays when it narrows the rows the gather has to move.
  s.tune = read_tuning();
  s.tf.assign(s.L, 0);
  for (int j = 0; j < s.L; ++j) {
    if (s.variant != GNNSTAGE_GCN) continue;
    const bool narrower = (size_t)s.dims[j + 1] * s.elt() < (size_t)s.dims[j] * s.level_elt(j);
    s.tf[j] = narrower ? 1 : 0;
    if (s.tune.order == 1) s.tf[j] = 0;
    if (s.tune.order == 2) s.tf[j] = 1;
  }
  if (d->row_ptr[0] != 0 || d->row_ptr[s.n] != s.nnz) { err = "row_ptr must start at 0 and end at nnz"; return false; }
  for (int64_t v = 0; v < s.n; ++v)
    if (d->row_ptr[v] > d->row_ptr[v + 1]) { err = "row_ptr must be non-decreasing"; return false; }
  return true;
}

Layout make_layout(const Shape &s, const HostDir &hf, const HostDir &hb, bool rank1) {
  const PlanCounts &f = hf.pc, &b = hb.pc;
  Layout l;
  Bump w;
  l.row_ptr = w.take(sizeof(int64_t) * (s.n + 1));
  l.pcol = w.take(sizeof(uint32_t) * hf.nnz);
  l.val = w.take(sizeof(float) * hf.nnz);
  l.t_ptr = w.take(sizeof(int64_t) * (s.n + 1));
  l.prow = w.take(sizeof(uint32_t) * hb.nnz);
  l.tval = w.take(sizeof(float) * hb.nnz);
  int64_t max_items = 0;
  for (int dir = 0; dir < 2; ++dir) {
    const HostDir &h = dir ? hb : hf;
    const bool on = h.dense();
    const size_t nb = on ? (size_t)h.dp.n_blocks() : 0, ne = on ? (size_t)h.padded_entries() : 0;
    const size_t ni = h.item_rb.size(), nl = on ? (size_t)h.pc.total_longs : 0;
    l.rem_ptr[dir] = w.take(on ? sizeof(int64_t) * (s.n + 1) : 0);
    l.d_blk_cb[dir] = w.take(sizeof(int32_t) * nb);
    l.d_blk_e0[dir] = w.take(on ? sizeof(int64_t) * (nb + 1) : 0);
    l.d_ent_pos[dir] = w.take(rank1 ? 0 : sizeof(uint16_t) * ne);
    l.d_ent_w[dir] = w.take(rank1 ? 0 : sizeof(uint32_t) * ne);
    l.d_colslot[dir] = w.take(on ? sizeof(uint32_t) * h.dp.colslot_vertex.size() : 0);
    l.d_tiles[dir] = w.take(rank1 ? 0 : sizeof(uint16_t) * nb * 2 * kDenseRB * kDenseCB);
    l.d_bits[dir] = w.take(rank1 ? sizeof(uint32_t) * nb * 256 : 0);
    l.d_colscale[dir] = w.take(on && rank1 ? sizeof(float) * h.dp.colslot_vertex.size() : 0);
    l.d_rowscale[dir] = w.take(on && rank1 ? sizeof(float) * (size_t)h.rowscale_off.back() : 0);
    l.d_item_rb[dir] = w.take(sizeof(int32_t) * ni);
    l.d_item_b0[dir] = w.take(sizeof(int64_t) * ni);
    l.d_item_nb[dir] = w.take(sizeof(int32_t) * ni);
    l.d_item_chunks[dir] = w.take(sizeof(ChunkMask) * ni);
    l.d_lr_dense0[dir] = w.take(sizeof(int32_t) * nl);
    l.d_lr_ndense[dir] = w.take(sizeof(int32_t) * nl);
    l.d_lr_item0[dir] = w.take(sizeof(int32_t) * nl);
    max_items = std::max(max_items, h.max_items);
  }
  l.dense_partial = w.take(sizeof(float) * (size_t)max_items * kDenseRB * 256);
  l.zero_row = w.take(max_items > 0 ? 512 : 0);
  l.f_task_row = w.take(sizeof(int32_t) * f.total_tasks);
  l.f_task_e0 = w.take(sizeof(int64_t) * f.total_tasks);
  l.f_task_ne = w.take(sizeof(int32_t) * f.total_tasks);
  l.f_task_slot = w.take(sizeof(int32_t) * f.total_tasks);
  l.f_lr_row = w.take(sizeof(int32_t) * f.total_longs);
  l.f_lr_slot0 = w.take(sizeof(int32_t) * f.total_longs);
  l.f_lr_n = w.take(sizeof(int32_t) * f.total_longs);
  l.b_task_row = w.take(sizeof(int32_t) * b.total_tasks);
  l.b_task_e0 = w.take(sizeof(int64_t) * b.total_tasks);
  l.b_task_ne = w.take(sizeof(int32_t) * b.total_tasks);
  l.b_task_slot = w.take(sizeof(int32_t) * b.total_tasks);
  l.b_lr_row = w.take(sizeof(int32_t) * b.total_longs);
  l.b_lr_slot0 = w.take(sizeof(int32_t) * b.total_longs);
  l.b_lr_n = w.take(sizeof(int32_t) * b.total_longs);
  l.f_slot_class = w.take((size_t)f.total_slots);
  l.b_slot_class = w.take((size_t)b.total_slots);
  int max_d = 0, max_ld = 0;
  size_t max_io = 0;
  for (int j = 0; j <= s.L; ++j) {
    max_d = std::max(max_d, s.dims[j]);
    max_ld = std::max(max_ld, s.ld[j]);
  }
  for (int j = 0; j < s.L; ++j) max_io = std::max(max_io, (size_t)s.dims[j] * s.dims[j + 1]);
  l.partial = w.take(sizeof(float) * (size_t)std::max(f.max_slots, b.max_slots) * max_d);
  const size_t elt = s.elt();
  l.Z.resize(s.L);
  l.dZ.resize(s.L);
  l.Wt.resize(s.L);
  l.Wn.resize(s.L);
  l.Tc.assign(s.L, 0);
  l.Th.assign(s.L, 0);
  l.dY.assign(s.L, 0);
  for (int j = 0; j < s.L && s.res(); ++j) {
    // ResGCN+: ReLU(LayerNorm(.)) of the current and of the historical rows, the saved aggregation, and the
    // gradient of the aggregation for ALL rows (the parameter gradient through historical rows needs it)
    l.Tc[j] = w.take((size_t)s.n * s.ld[j] * elt);
    l.Th[j] = w.take((size_t)s.n * s.ld[j] * elt);
    l.Z[j] = w.take((size_t)s.n * s.ld[j] * elt);
    l.dZ[j] = w.take((size_t)s.n * s.ld[j] * elt);
  }
  if (s.res()) {
    l.res_dr = w.take((size_t)s.max_rows() * max_ld * elt);
    l.ln_partial = w.take(sizeof(float) * (size_t)(kLnMaxWaves / 4) * 2 * max_d);
  }
  for (int j = 0; j < s.L && !s.res(); ++j) {
    if (s.tf[j]) {
      // transform-first layer: transformed current / historical rows, and the masked upstream gradient
      l.Z[j] = 0;
      l.Tc[j] = w.take((size_t)s.n * s.ld[j + 1] * elt);
      l.Th[j] = w.take((size_t)s.n * s.ld[j + 1] * elt);
      l.dZ[j] = w.take((size_t)s.n * s.ld[j + 1] * elt);
    } else {
      l.Z[j] = w.take((size_t)s.n * s.ld[j] * elt);
      l.dZ[j] = (j == 0 && !s.need_input_grad) ? 0 : w.take((size_t)s.n * s.ld[j] * elt);
      if (s.defer_wgrad()) l.dY[j] = w.take((size_t)s.n * s.ld[j + 1] * elt);
    }
  }
  for (int j = 0; j < s.L; ++j) {
    l.Wt[j] = w.take((size_t)s.dims[j + 1] * s.ld[j] * elt);
    l.Wn[j] = w.take((size_t)s.dims[j] * s.ld[j + 1] * elt);
  }
  if (s.sage()) {
    l.Wt_self.resize(s.L);
    l.Wn_self.resize(s.L);
    for (int j = 0; j < s.L; ++j) {
      l.Wt_self[j] = w.take((size_t)s.dims[j + 1] * s.ld[j] * elt);
      l.Wn_self[j] = w.take((size_t)s.dims[j] * s.ld[j + 1] * elt);
    }
    l.self_fwd = w.take(sizeof(float) * (size_t)s.max_rows() * max_ld);
    l.self_bwd = w.take((size_t)s.max_rows() * max_ld * elt);
  }
  l.G[0] = w.take((size_t)s.max_rows() * max_ld * elt);
  l.G[1] = w.take((size_t)s.max_rows() * max_ld * elt);
  l.gemm_partial = w.take(sizeof(float) * kMaxSplits * max_io);
  l.bias_partial = w.take(sizeof(float) * kMaxSplits * max_d);
  l.total = w.off;
  return l;
}

struct Profiler {
  uint32_t kinds = 0;  // bit k set: launches of kind k are timed
  int n_layers = 0;  // slot n_layers collects launches that belong to no layer
  struct Rec { int kind, layer; hipEvent_t a, b; };
  std::vector<Rec> recs;
  std::vector<hipEvent_t> free_events;
  std::vector<double> ms;          // [kind][layer]
  std::vector<int64_t> launches;   // [kind][layer]
  void init(int L) {
    n_layers = L;
    ms.assign((size_t)GNNSTAGE_NKINDS * (L + 1), 0.0);
    launches.assign((size_t)GNNSTAGE_NKINDS * (L + 1), 0);
  }
  hipEvent_t get() {
    if (!free_events.empty()) {
      hipEvent_t e = free_events.back();
      free_events.pop_back();
      return e;
    }
    hipEvent_t e = nullptr;
    // timing only: no system-scope fence when the event completes (the default event makes every write of the
    // stream visible to the host, which costs a launch of a few microseconds about as much as the launch itself)
    (void)hipEventCreateWithFlags(&e, hipEventDisableSystemFence);
    return e;
  }
  void collect() {
    for (auto &r : recs) {
      float t = 0.f;
      if (hipEventElapsedTime(&t, r.a, r.b) == hipSuccess) {
        ms[(size_t)r.kind * (n_layers + 1) + r.layer] += t;
        launches[(size_t)r.kind * (n_layers + 1) + r.layer] += 1;
      }
      free_events.push_back(r.a);
      free_events.push_back(r.b);
    }
    recs.clear();
  }
  void destroy() {
    collect();
    for (auto e : free_events) (void)hipEventDestroy(e);
    free_events.clear();
  }
};

}  // namespace

struct gnnstage {
  Shape s;
  Layout lay;
  int vbits = 0;
  float alpha = 0.f;
  std::vector<float> beta;
  // caller-owned device buffers
  std::vector<void *> W, bias, cur, hist;
  std::vector<float *> dW, dbias;
  const void *h0 = nullptr;
  std::vector<const float *> ln_g, ln_b;  // ResGCN+: LayerNorm parameters and their gradients
  std::vector<float *> d_ln_g, d_ln_b;
  float ln_eps = 1e-5f;
  float dropout_p = 0.f;      // ResGCN+: between ReLU and the convolution; GCN, GraphSage: on every layer's output
  uint64_t dropout_seed = 0;  // of the current pass
  // What the setters wrote.  A pass latches both at its first forward call and keeps them until its last backward
  // call, so that the backward pass redraws exactly the decisions of its forward pass whatever the caller sets
  // in between.
  float next_dropout_p = 0.f;
  uint64_t next_dropout_seed = 0;
  // GCN, GraphSage: the stored output of a layer is the value after dropout; a positive one passed ReLU and dropout,
  // so every ReLU mask of the backward pass also scales by 1 / (1 - rate)
  bool output_dropout() const { return dropout_p > 0.f && (s.variant == GNNSTAGE_GCN || s.variant == GNNSTAGE_SAGE); }
  float mask_scale() const { return output_dropout() ? (float)(1.0 / (1.0 - (double)dropout_p)) : 1.f; }
  // the dropout of layer j for a launch whose first row is vertex u0
  LnDropout dropout(int j, int64_t u0) const {
    LnDropout dp{};
    if (dropout_p > 0.f) {
      uint64_t z = dropout_seed + (uint64_t)(j + 1) * 0x9E3779B97F4A7C15ull;  // SplitMix64 output for that state
      z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
      z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
      dp.key = z ^ (z >> 31);
      dp.threshold = (uint32_t)std::ceil((double)dropout_p * 16777216.0);
      dp.scale = (float)(1.0 / (1.0 - (double)dropout_p));
      dp.u0 = u0;
    }
    return dp;
  }
  void *grad_in = nullptr;
  float *grad_h0 = nullptr;
  char *ws = nullptr;
  // host copies for the diagnostics
  std::vector<int64_t> h_row_ptr;
  std::vector<uint32_t> h_pcol;
  // schedules
  std::vector<TaskList> ftasks, btasks;
  bool dense_on[2] = {false, false};  // dense blocks per direction (0 forward, 1 transposed)
  int64_t dense_entries[2] = {0, 0};  // entries that live in dense blocks
  bool dense_rank1 = false;           // their weights are kept as pattern bits and row / column scales
  std::vector<int64_t> rowscale_off[2];
  int n_classes = 1;
  // pass state (Section 3.3: V_processed, and its backward twin)
  std::vector<int32_t> order;
  ChunkMask fmask{}, bmask{};
  int n_bwd = 0;
  bool cur_stale = false;  // the levels traded places and no complete pass has rewritten the current ones yet
  std::vector<char> wgrad_pending;  // per chunk: its backward call ran, its rows' weight-gradient products are still owed
  std::string err;
  Profiler prof;

  template <typename T>
  T *at(size_t off) const { return reinterpret_cast<T *>(ws + off); }
  int level_dtype(int j) const { return (j == 0 && s.level0_f32) ? DT_F32 : (s.dtype == GNNSTAGE_BF16 ? DT_BF16 : DT_F32); }
  int cdtype() const { return s.dtype == GNNSTAGE_BF16 ? DT_BF16 : DT_F32; }
  size_t level_elt(int j) const { return level_dtype(j) == DT_BF16 ? 2 : 4; }
};

namespace {

int fail(gnnstage *st, int code, const std::string &msg) {
  if (st) st->err = msg; else g_create_error = msg;
  return code;
}

struct Timed {
  gnnstage *st;
  hipStream_t s;
  int kind, layer;
  hipEvent_t a = nullptr, b = nullptr;
  Timed(gnnstage *st_, hipStream_t s_, int kind_, int layer_ = -1)
      : st(st_), s(s_), kind(kind_), layer(layer_ < 0 ? st_->prof.n_layers : layer_) {
    if ((st->prof.kinds >> kind) & 1u) {
      a = st->prof.get();
      b = st->prof.get();
      (void)hipEventRecord(a, s);
    }
  }
  ~Timed() {
    if (a != nullptr) {
      (void)hipEventRecord(b, s);
      st->prof.recs.push_back({kind, layer, a, b});
    }
  }
};

#define HIP_TRY(st, expr)                                                                            \
  do {                                                                                               \
    const int e_ = (int)(expr);                                                                      \
    if (e_ != 0)                                                                                     \
      return fail(st, GNNSTAGE_EHIP, std::string(#expr) + ": " + hipGetErrorString((hipError_t)e_)); \
  } while (0)

void mask_set(ChunkMask &m, int c) { m.w[c >> 6] |= 1ull << (c & 63); }

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// XCD assignment of the class sections for one launch.  `drop` = the launch skips unselected entries:
// a class with no entry from a chunk in the mask has no work and is not served at all.  Every class gets
// a cost (a fixed part per task, one unit per gathered entry, a small part per entry that is read and
// dropped), and the groups of the active classes are dealt to the 8 XCDs like water into buckets of equal
// cost, a class being split between neighbouring XCDs where a bucket boundary falls inside it.
void assign_xcds(const gnnstage *st, const TaskList &t, const ChunkMask &mask, bool drop, SpmmArgs &a) {
  const int C = t.n_classes, K = st->s.K;
  a.tail_task0 = t.cls_off[C];
  a.slot_class = t.slot_class;
  a.active_classes = 0;
  a.all_classes_active = 1;
  a.n_class_blocks = 0;
  int groups[kMaxClasses];
  double unit[kMaxClasses];  // cost of one group of four tasks
  double total = 0;
  for (int x = 0; x < 8; ++x)
    for (int sgm = 0; sgm < kMaxSegs; ++sgm) a.seg_cls[x][sgm] = a.seg_g0[x][sgm] = a.seg_cnt[x][sgm] = 0;
  for (int q = 0; q < kMaxClasses; ++q) {
    a.cls_task0[q] = a.cls_ntasks[q] = 0;
    groups[q] = 0;
    unit[q] = 0;
    if (q >= C) continue;
    a.cls_task0[q] = (int32_t)t.cls_off[q];
    a.cls_ntasks[q] = (int32_t)(t.cls_off[q + 1] - t.cls_off[q]);
    int64_t kept = 0, all = 0;
    for (int c = 0; c < K; ++c) {
      const int64_t e = t.cls_chunk_entries[(size_t)q * K + c];
      all += e;
      if (!drop || mask_test(mask, c)) kept += e;
    }
    const bool on = a.cls_ntasks[q] > 0 && kept > 0;
    if (!on) a.all_classes_active = 0;
    if (!on) continue;
    a.active_classes |= 1u << q;
    groups[q] = (a.cls_ntasks[q] + 3) / 4;
    const double cost = 32.0 * a.cls_ntasks[q] + (double)kept + 0.125 * (double)(all - kept);
    unit[q] = cost / groups[q];
    total += cost;
  }
  if (total == 0) return;
  const double quota = total / 8;
  int x = 0, nseg = 0, most = 0, load = 0;
  double used = 0;
  bool fits = true;
  for (int q = 0; q < C && fits; ++q) {
    int g = 0;
    while (g < groups[q]) {
      if (x < 7 && (used >= quota - 0.5 * unit[q] || nseg == kMaxSegs)) {
        ++x;
        used = 0;
        nseg = 0;
        load = 0;
      }
      if (nseg == kMaxSegs) {  // many tiny classes left for the last XCD
        fits = false;
        break;
      }
      int take = groups[q] - g;
      if (x < 7) {
        const int room = (int)((quota - used) / unit[q] + 0.5);
        take = std::min(take, std::max(room, 1));
      }
      a.seg_cls[x][nseg] = q;
      a.seg_g0[x][nseg] = g;
      a.seg_cnt[x][nseg] = take;
      ++nseg;
      g += take;
      used += take * unit[q];
      load += take;
      most = std::max(most, load);
    }
  }
  if (!fits) {  // fallback that always fits: class q goes whole to XCD q % 8 (at most 4 segments each)
    most = 0;
    int cnt[8] = {0, 0, 0, 0, 0, 0, 0, 0}, ld[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int xx = 0; xx < 8; ++xx)
      for (int sgm = 0; sgm < kMaxSegs; ++sgm) a.seg_cls[xx][sgm] = a.seg_g0[xx][sgm] = a.seg_cnt[xx][sgm] = 0;
    for (int q = 0; q < C; ++q) {
      if (groups[q] == 0) continue;
      const int xx = q & 7;
      a.seg_cls[xx][cnt[xx]] = q;
      a.seg_g0[xx][cnt[xx]] = 0;
      a.seg_cnt[xx][cnt[xx]] = groups[q];
      ++cnt[xx];
      ld[xx] += groups[q];
      most = std::max(most, ld[xx]);
    }
  }
  a.n_class_blocks = 8 * most;
}

SpmmArgs base_spmm(const gnnstage *st, bool transposed, int chunk) {
  SpmmArgs a{};
  const TaskList &t = transposed ? st->btasks[chunk] : st->ftasks[chunk];
  a.pidx = st->at<uint32_t>(transposed ? st->lay.prow : st->lay.pcol);
  a.val = st->at<float>(transposed ? st->lay.tval : st->lay.val);
  a.task_row = t.task_row;
  a.task_e0 = t.task_e0;
  a.task_ne = t.task_ne;
  a.task_slot = t.task_slot;
  a.n_tasks = t.n_tasks;
  a.n_short = t.n_short;
  a.lr_row = t.lr_row;
  a.lr_slot0 = t.lr_slot0;
  a.lr_nslots = t.lr_nslots;
  a.n_long = t.n_long;
  a.partial = st->at<float>(st->lay.partial);
  a.vbits = st->vbits;
  a.force_valu = st->s.tune.spmm_valu ? 1 : 0;
  a.unroll = st->s.tune.spmm_unroll;
  a.mask = transposed ? st->bmask : st->fmask;
  const int dir = transposed ? 1 : 0;
  if (st->dense_on[dir]) {
    a.lr_dense0 = t.lr_dense0;
    a.lr_ndense = t.lr_ndense;
    a.lr_item0 = t.lr_item0;
    a.item_chunks = st->at<ChunkMask>(st->lay.d_item_chunks[dir]) + t.item0;
    a.dense_partial = st->at<float>(st->lay.dense_partial);
  }
  assign_xcds(st, t, a.mask, transposed, a);  // every transposed launch drops unselected entries
  return a;
}

// aggregation kernel and (when the chunk has long rows) the reduce of their pieces, timed apart
// (with dense blocks: their kernel first, timed together with the sparse kernel)
int run_spmm(gnnstage *st, const SpmmArgs &a_in, bool transposed, int chunk, int src_dtype, int out_dtype,
             hipStream_t stream, int kind, int layer) {
  SpmmArgs a = a_in;
  a.drop_unselected = a.src_unsel == nullptr ? 1 : 0;
  const int dir = transposed ? 1 : 0;
  const TaskList &t = transposed ? st->btasks[chunk] : st->ftasks[chunk];
  {
    Timed tm(st, stream, kind, layer);
    if (st->dense_on[dir] && t.n_items > 0) {
      if (src_dtype != DT_BF16 || (a.d != 128 && a.d != 256) || a.src_ld != a.d) return hipErrorInvalidValue;
      const Layout &lay = st->lay;
      DenseArgs da{};
      da.item_rb = st->at<int32_t>(lay.d_item_rb[dir]) + t.item0;
      da.item_b0 = st->at<int64_t>(lay.d_item_b0[dir]) + t.item0;
      da.item_nb = st->at<int32_t>(lay.d_item_nb[dir]) + t.item0;
      da.item_chunks = st->at<ChunkMask>(lay.d_item_chunks[dir]) + t.item0;
      da.n_items = t.n_items;
      da.blk_cb = st->at<int32_t>(lay.d_blk_cb[dir]);
      if (st->dense_rank1) {
        da.bits = st->at<uint32_t>(lay.d_bits[dir]);
        da.colscale = st->at<float>(lay.d_colscale[dir]);
        da.rowscale = st->at<float>(lay.d_rowscale[dir]) + st->rowscale_off[dir][(size_t)chunk];
      } else {
        da.tiles = st->at<bf16_t>(lay.d_tiles[dir]);
      }
      da.zero_row = st->at<char>(lay.zero_row);
      da.colslot = st->at<uint32_t>(lay.d_colslot[dir]);
      da.src_sel = a.src_sel;
      da.src_unsel = a.src_unsel;
      da.d = a.d;
      da.src_ld = a.src_ld;
      da.vbits = a.vbits;
      da.mask = a.mask;
      da.partial = st->at<float>(lay.dense_partial);
      const int e = launch_spmm_dense(da, stream);
      if (e != 0) return e;
    }
    const int e = launch_spmm(a, src_dtype, out_dtype, stream);
    if (e != 0) return e;
  }
  if (a.n_long > 0) {
    Timed tm(st, stream, 7, layer);
    return launch_spmm_reduce(a, src_dtype, out_dtype, stream);
  }
  return 0;
}

// After the last backward call of a pass: the history-side weight gradient of every transform-first
// layer, dW += hist^T (A_hat^T dY), chunk by chunk through the gradient scratch rows.
int finish_transform_first(gnnstage *st, hipStream_t stream) {
  const Shape &s = st->s;
  const int cd = st->cdtype();
  ChunkMask all{};
  for (int c = 0; c < s.K; ++c) mask_set(all, c);
  char *dT = st->at<char>(st->lay.G[0]);
  for (int j = 0; j < s.L; ++j) {
    if (!s.tf[j]) continue;
    for (int c = 0; c < s.K; ++c) {
      const int64_t row0 = s.chunk_ptr[c], M = s.chunk_ptr[c + 1] - row0;
      if (M == 0) continue;
      SpmmArgs a = base_spmm(st, true, c);
      a.mask = all;
      assign_xcds(st, st->btasks[c], all, true, a);
      a.src_sel = st->at<char>(st->lay.dZ[j]);
      a.src_unsel = nullptr;
      a.d = s.dims[j + 1];
      a.src_ld = s.ld[j + 1];
      a.out = dT;
      a.out_ld = s.ld[j + 1];
      a.out_row0 = row0;
      a.epilogue = SPMM_PLAIN;
      HIP_TRY(st, run_spmm(st, a, true, c, cd, cd, stream, 2, j));
      Timed t(st, stream, 4, j);
      GemmTnArgs w{};
      w.wide_min_rows = st->s.tune.gemm_wide_min_rows;
      w.A = static_cast<const char *>(st->hist[j]) + (size_t)row0 * s.dims[j] * st->level_elt(j);
      w.a_dtype = st->level_dtype(j);
      w.lda = s.dims[j];
      w.B = dT;
      w.ldb = s.ld[j + 1];
      w.M = (int)M;
      w.I = s.dims[j];
      w.O = s.dims[j + 1];
      w.scale = 1.f;
      w.dW = st->dW[j];
      w.partial = st->at<float>(st->lay.gemm_partial);
      w.max_splits = kMaxSplits;
      HIP_TRY(st, launch_gemm_tn(w, cd, stream));
    }
  }
  return GNNSTAGE_OK;
}

// ---- ResGCN+ (LayerNorm -> ReLU -> GCN convolution, plus the residual) ------------------------------------
// Layer j: r_u = ReLU(LayerNorm_j(h_u)) on whichever row of u is read (current or historical),
// z_v = sum_u A_vu r_u, h'_v = h_v + z_v W_j + b_j.  The activated rows are tables: Rh = f(hist[j]) once per
// pass, Rc[C_k] = f(cur[j][C_k]) when the chunk is computed.
int res_pass_start(gnnstage *st, hipStream_t stream) {
  const Shape &s = st->s;
  const int cd = st->cdtype();
  for (int j = 0; j < s.L; ++j) {
    Timed t(st, stream, 1, j);
    HIP_TRY(st, launch_ln_relu(st->hist[j], st->level_dtype(j), s.dims[j], st->ln_g[j], st->ln_b[j], st->ln_eps, s.n, s.dims[j],
                               st->at<char>(st->lay.Th[j]), cd, s.ld[j], st->dropout(j, 0), stream));
  }
  return GNNSTAGE_OK;
}

int res_forward_chunk(gnnstage *st, int k, hipStream_t stream) {
  const Shape &s = st->s;
  const int cd = st->cdtype();
  const size_t celt = s.elt();
  const int64_t row0 = s.chunk_ptr[k], M = s.chunk_ptr[k + 1] - row0;
  for (int j = 0; j < s.L; ++j) {
    const bool shared = st->hist[j] == st->cur[j];  // the level never changes: one activated table serves both
    char *Rh = st->at<char>(st->lay.Th[j]);
    char *Rc = shared ? Rh : st->at<char>(st->lay.Tc[j]);
    const char *xrows = static_cast<const char *>(st->cur[j]) + (size_t)row0 * s.dims[j] * st->level_elt(j);
    if (!shared) {
      Timed t(st, stream, 1, j);
      HIP_TRY(st, launch_ln_relu(xrows, st->level_dtype(j), s.dims[j], st->ln_g[j], st->ln_b[j], st->ln_eps, M, s.dims[j],
                                 Rc + (size_t)row0 * s.ld[j] * celt, cd, s.ld[j], st->dropout(j, row0), stream));
    }
    char *Zj = st->at<char>(st->lay.Z[j]);
    {
      SpmmArgs a = base_spmm(st, false, k);
      a.src_sel = Rc;
      a.src_unsel = Rh;
      a.d = s.dims[j];
      a.src_ld = s.ld[j];
      a.out = Zj;
      a.out_ld = s.ld[j];
      a.out_row0 = 0;
      a.epilogue = SPMM_PLAIN;
      HIP_TRY(st, run_spmm(st, a, false, k, cd, cd, stream, 0, j));
    }
    {
      Timed t(st, stream, 1, j);
      GemmNtArgs g{};
      g.ws_min_rows = st->s.tune.gemm_ws_min_rows;
      g.A = Zj + (size_t)row0 * s.ld[j] * celt;
      g.a_dtype = cd;
      g.lda = s.ld[j];
      g.Bt = st->at<char>(st->lay.Wt[j]);
      g.ldb = s.ld[j];
      g.M = (int)M;
      g.N = s.dims[j + 1];
      g.K = s.dims[j];
      g.Kp = s.ld[j];
      g.epilogue = EPI_RES;
      g.bias = static_cast<const float *>(st->bias[j]);
      g.aux = xrows;
      g.aux_dtype = st->level_dtype(j);
      g.aux_ld = s.dims[j];
      g.out = static_cast<char *>(st->cur[j + 1]) + (size_t)row0 * s.dims[j + 1] * celt;
      g.out_dtype = cd;
      g.out_ld = s.dims[j + 1];
      HIP_TRY(st, launch_gemm_nt(g, cd, stream));
    }
  }
  return GNNSTAGE_OK;
}

// After the last backward chunk: the LayerNorm of layer j was also applied to the historical rows, so its
// parameters receive gradient through every edge whose reader saw the historical row of u: the readers whose
// chunk came before u's chunk in the forward order.
int res_backward_finish(gnnstage *st, hipStream_t stream) {
  const Shape &s = st->s;
  const int cd = st->cdtype();
  const size_t celt = s.elt();
  char *dR = st->at<char>(st->lay.res_dr);
  ChunkMask earlier{};  // chunks in front of the current one, grown along the forward order
  for (size_t pos = 0; pos < st->order.size(); ++pos) {
    const int c = st->order[pos];
    const int64_t row0 = s.chunk_ptr[c], M = s.chunk_ptr[c + 1] - row0;
    if (pos > 0 && M > 0) {
      for (int j = 0; j < s.L; ++j) {
        SpmmArgs a = base_spmm(st, true, c);
        a.mask = earlier;
        assign_xcds(st, st->btasks[c], earlier, true, a);
        a.src_sel = st->at<char>(st->lay.dZ[j]);
        a.src_unsel = nullptr;
        a.d = s.dims[j];
        a.src_ld = s.ld[j];
        a.out = dR;
        a.out_ld = s.ld[j];
        a.out_row0 = row0;
        a.epilogue = SPMM_PLAIN;
        HIP_TRY(st, run_spmm(st, a, true, c, cd, cd, stream, 2, j));
        Timed t(st, stream, 4, j);
        const char *xrows = static_cast<const char *>(st->hist[j]) + (size_t)row0 * s.dims[j] * st->level_elt(j);
        HIP_TRY(st, launch_ln_relu_backward(xrows, st->level_dtype(j), s.dims[j], st->ln_g[j], st->ln_b[j], st->ln_eps, dR, cd, s.ld[j],
                                            nullptr, cd, 0, M, s.dims[j], nullptr, cd, 0, st->at<float>(st->lay.ln_partial),
                                            st->d_ln_g[j], st->d_ln_b[j], st->dropout(j, row0), stream));
      }
    }
    mask_set(earlier, c);
  }
  return GNNSTAGE_OK;
}

int res_backward_chunk(gnnstage *st, int k, const void *grad_out_rows, hipStream_t stream) {
  const Shape &s = st->s;
  const int cd = st->cdtype();
  const size_t celt = s.elt();
  const int64_t row0 = s.chunk_ptr[k], M = s.chunk_ptr[k + 1] - row0;
  char *G[2] = {st->at<char>(st->lay.G[0]), st->at<char>(st->lay.G[1])};
  char *dR = st->at<char>(st->lay.res_dr);
  float *gemm_partial = st->at<float>(st->lay.gemm_partial);
  float *bias_partial = st->at<float>(st->lay.bias_partial);
  int gi = 0;
  if (M > 0) {
    Timed t(st, stream, 6);  // no activation after the convolution: dY of the top layer is the upstream gradient
    HIP_TRY(st, launch_copy_rows(grad_out_rows, s.dims[s.L], G[gi], s.ld[s.L], M, s.dims[s.L], cd, stream));
  }
  for (int j = s.L - 1; j >= 0 && M > 0; --j) {
    const char *dY = G[gi];
    const bool fuse_bias = cd == DT_BF16;
    if (!fuse_bias) {
      Timed t(st, stream, 4, j);
      HIP_TRY(st, launch_colsum_add(dY, cd, s.ld[j + 1], (int)M, s.dims[j + 1], bias_partial, kMaxSplits, st->dbias[j], stream));
    }
    {
      Timed t(st, stream, 4, j);
      GemmTnArgs w{};
      w.wide_min_rows = st->s.tune.gemm_wide_min_rows;
      w.A = st->at<char>(st->lay.Z[j]) + (size_t)row0 * s.ld[j] * celt;
      w.a_dtype = cd;
      w.lda = s.ld[j];
      w.B = dY;
      w.ldb = s.ld[j + 1];
      w.M = (int)M;
      w.I = s.dims[j];
      w.O = s.dims[j + 1];
      w.scale = 1.f;
      w.dW = st->dW[j];
      w.partial = gemm_partial;
      w.max_splits = kMaxSplits;
      if (fuse_bias) {
        w.dbias = st->dbias[j];
        w.bias_partial = bias_partial;
      }
      HIP_TRY(st, launch_gemm_tn(w, cd, stream));
    }
    char *dZj = st->at<char>(st->lay.dZ[j]);
    {
      Timed t(st, stream, 3, j);
      GemmNtArgs g{};
      g.ws_min_rows = st->s.tune.gemm_ws_min_rows;
      g.A = dY;
      g.a_dtype = cd;
      g.lda = s.ld[j + 1];
      g.Bt = st->at<char>(st->lay.Wn[j]);
      g.ldb = s.ld[j + 1];
      g.M = (int)M;
      g.N = s.dims[j];
      g.K = s.dims[j + 1];
      g.Kp = s.ld[j + 1];
      g.epilogue = EPI_PLAIN;
      g.out = dZj + (size_t)row0 * s.ld[j] * celt;
      g.out_dtype = cd;
      g.out_ld = s.ld[j];
      HIP_TRY(st, launch_gemm_nt(g, cd, stream));
    }
    {
      SpmmArgs a = base_spmm(st, true, k);
      a.src_sel = dZj;
      a.src_unsel = nullptr;  // Section 3.4: nothing flows back from unprocessed vertices
      a.d = s.dims[j];
      a.src_ld = s.ld[j];
      a.out = dR;
      a.out_ld = s.ld[j];
      a.out_row0 = row0;
      a.epilogue = SPMM_PLAIN;
      HIP_TRY(st, run_spmm(st, a, true, k, cd, cd, stream, 2, j));
    }
    {
      // back through ReLU and LayerNorm of the chunk's own (current) rows, plus the residual branch
      Timed t(st, stream, 4, j);
      const char *xrows = static_cast<const char *>(st->cur[j]) + (size_t)row0 * s.dims[j] * st->level_elt(j);
      void *out = nullptr;
      int out_ld = 0;
      if (j > 0) {
        out = G[gi ^ 1];
        out_ld = s.ld[j];
      } else if (s.need_input_grad) {
        out = static_cast<char *>(st->grad_in) + (size_t)row0 * s.dims[0] * st->level_elt(0);
        out_ld = s.dims[0];
      }
      HIP_TRY(st, launch_ln_relu_backward(xrows, st->level_dtype(j), s.dims[j], st->ln_g[j], st->ln_b[j], st->ln_eps, dR, cd, s.ld[j], dY,
                                          cd, s.ld[j + 1], M, s.dims[j], out, st->level_dtype(j), out_ld,
                                          st->at<float>(st->lay.ln_partial), st->d_ln_g[j], st->d_ln_b[j], st->dropout(j, row0), stream));
    }
    gi ^= 1;
  }
  if (st->n_bwd == s.K) return res_backward_finish(st, stream);
  return GNNSTAGE_OK;
}

}  // namespace

extern "C" int gnnstage_version(void) { return 100; }

extern "C" int64_t gnnstage_dense_entries(const gnnstage_t *st, int32_t transposed) {
  if (!st) return GNNSTAGE_EINVAL;
  return st->dense_entries[transposed ? 1 : 0];
}

extern "C" const char *gnnstage_last_error(const gnnstage_t *st) { return st ? st->err.c_str() : g_create_error.c_str(); }

namespace {
// transposed index and the per-direction plans: what both the size query and create need
struct HostPlan {
  std::vector<int64_t> t_ptr, t_edge;
  std::vector<int32_t> t_row;
  HostDir f, b;
};

int make_host_plan(const gnnstage_desc *d, const Shape &s, bool want_edge, HostPlan &hp, std::string &err) {
  if (s.nnz > 0 && !d->col_idx) {
    err = "col_idx is NULL";
    return GNNSTAGE_EINVAL;
  }
  hp.t_ptr.assign((size_t)s.n + 1, 0);
  hp.t_row.resize((size_t)s.nnz);
  if (want_edge) hp.t_edge.resize((size_t)s.nnz);
  if (gnnstage_plan_transpose(s.n, d->row_ptr, d->col_idx, hp.t_ptr.data(), hp.t_row.data(),
                              want_edge ? hp.t_edge.data() : nullptr) != GNNSTAGE_OK) {
    err = "col_idx is NULL or has an entry outside [0, n_vertices)";
    return GNNSTAGE_EINVAL;
  }
  const bool dense = s.dense_ok();
  if (!make_host_dir(s.tune, d->row_ptr, d->col_idx, s.n, s.chunk_ptr, s.classes(), s.hot(), want_edge, dense, s.dense_width(), hp.f) ||
      !make_host_dir(s.tune, hp.t_ptr.data(), hp.t_row.data(), s.n, s.chunk_ptr, s.classes(), s.hot(), want_edge, dense, s.dense_width(), hp.b)) {
    err = "cannot plan the aggregation";
    return GNNSTAGE_EINVAL;
  }
  return GNNSTAGE_OK;
}

uint16_t bf16_bits_rne(float f) {  // finite inputs: round to nearest even, as the device conversion does
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
float bf16_bits_to_f32(uint16_t h) {
  const uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}
}  // namespace

extern "C" size_t gnnstage_workspace_size(const gnnstage_desc *desc) try {
  Shape s;
  std::string err;
  if (!read_shape(desc, s, err)) {
    g_create_error = err;
    return 0;
  }
  HostPlan hp;
  if (make_host_plan(desc, s, false, hp, err) != GNNSTAGE_OK) {
    g_create_error = err;
    return 0;
  }
  return make_layout(s, hp.f, hp.b, desc->edge_val == nullptr).total;
}
GNNSTAGE_GUARD_SIZE

extern "C" int gnnstage_create(const gnnstage_desc *d, gnnstage_t **out) try {
  if (!out) return fail(nullptr, GNNSTAGE_EINVAL, "out is NULL");
  *out = nullptr;
  Shape s;
  std::string err;
  if (!read_shape(d, s, err)) return fail(nullptr, GNNSTAGE_EINVAL, err);
  // The library computes the weights itself: w(v, u) = s_row(v) s_col(u), which the dense blocks keep as patterns.
  const bool rank1 = d->edge_val == nullptr;
  // GraphSage without weights: the mean aggregator, 1 / |N(v)| on every entry of row v; the sparse kernels take
  // it from here on like weights the caller gave
  std::vector<float> mean_val;
  gnnstage_desc with_mean;
  if (s.sage() && !d->edge_val && d->row_ptr) {
    mean_val.resize((size_t)s.nnz);
    for (int64_t v = 0; v < s.n; ++v) {
      const int64_t e0 = d->row_ptr[v], e1 = d->row_ptr[v + 1];
      if (e0 < 0 || e1 < e0 || e1 > s.nnz) return fail(nullptr, GNNSTAGE_EINVAL, "row_ptr is not a valid CSR pointer array");
      for (int64_t e = e0; e < e1; ++e) mean_val[(size_t)e] = 1.f / (float)(e1 - e0);
    }
    with_mean = *d;
    with_mean.edge_val = mean_val.data();
    d = &with_mean;
  }
  if (!d->W || !d->cur || !d->hist) return fail(nullptr, GNNSTAGE_EINVAL, "W, cur and hist must not be NULL");
  if (!d->dW) return fail(nullptr, GNNSTAGE_EINVAL, "dW must not be NULL");
  if (s.has_bias() && (!d->bias || !d->dbias)) return fail(nullptr, GNNSTAGE_EINVAL, "GCN and GraphSage need bias and dbias");
  if (s.variant == GNNSTAGE_GCNII && (!d->beta || !d->h0)) return fail(nullptr, GNNSTAGE_EINVAL, "GCNII needs beta and h0");
  if (s.res()) {
    if (!d->ln_gamma || !d->ln_beta || !d->d_ln_gamma || !d->d_ln_beta)
      return fail(nullptr, GNNSTAGE_EINVAL, "ResGCN+ needs ln_gamma, ln_beta and their gradient arrays");
    for (int j = 0; j < s.L; ++j)
      if (!d->ln_gamma[j] || !d->ln_beta[j] || !d->d_ln_gamma[j] || !d->d_ln_beta[j])
        return fail(nullptr, GNNSTAGE_EINVAL, "a LayerNorm parameter pointer is NULL");
    if (!(d->ln_eps > 0.f)) return fail(nullptr, GNNSTAGE_EINVAL, "ln_eps must be positive");
  }
  if (!(d->dropout_p >= 0.f && d->dropout_p < 1.f)) return fail(nullptr, GNNSTAGE_EINVAL, "dropout_p must be in [0, 1)");
  if (d->dropout_p > 0.f && s.variant == GNNSTAGE_GCNII) return fail(nullptr, GNNSTAGE_EINVAL, "no dropout in GCNII layers");
  if (s.need_input_grad && !d->grad_in) return fail(nullptr, GNNSTAGE_EINVAL, "need_input_grad set but grad_in is NULL");
  if (!d->workspace || (reinterpret_cast<uintptr_t>(d->workspace) & (kAlign - 1)))
    return fail(nullptr, GNNSTAGE_EINVAL, "workspace must be a 256-byte aligned device pointer");
  for (int j = 0; j <= s.L; ++j) {
    if (!d->cur[j] || !aligned16(d->cur[j])) return fail(nullptr, GNNSTAGE_EINVAL, "cur[j] NULL or not 16-byte aligned");
    if (j < s.L) {
      if (!d->hist[j] || !aligned16(d->hist[j])) return fail(nullptr, GNNSTAGE_EINVAL, "hist[j] NULL or not 16-byte aligned");
      if (!d->W[j] || !d->dW[j]) return fail(nullptr, GNNSTAGE_EINVAL, "W[j] / dW[j] NULL");
      if (s.has_bias() && (!d->bias[j] || !d->dbias[j])) return fail(nullptr, GNNSTAGE_EINVAL, "bias[j] / dbias[j] NULL");
    }
  }
  if ((d->h0 && !aligned16(d->h0)) || (d->grad_in && !aligned16(d->grad_in)))
    return fail(nullptr, GNNSTAGE_EINVAL, "h0 / grad_in not 16-byte aligned");

  // ---- host planning -------------------------------------------------------------------
  HostPlan hp;
  int rc = make_host_plan(d, s, d->edge_val != nullptr, hp, err);
  if (rc != GNNSTAGE_OK) return fail(nullptr, rc, err);
  const std::vector<int64_t> &t_ptr = hp.t_ptr, &t_edge = hp.t_edge;
  int vbits = 0;
  std::vector<uint32_t> pcol((size_t)hp.f.nnz), prow((size_t)hp.b.nnz);
  rc = gnnstage_plan_pack(s.n, hp.f.nnz, hp.f.idx, s.K, s.chunk_ptr.data(), pcol.data(), &vbits);
  if (rc == GNNSTAGE_ENOTSUP)
    return fail(nullptr, rc, "vertex-id bits + chunk-id bits exceed the 32-bit packed index word");
  if (rc != GNNSTAGE_OK) return fail(nullptr, rc, "cannot pack column indices");
  rc = gnnstage_plan_pack(s.n, hp.b.nnz, hp.b.idx, s.K, s.chunk_ptr.data(), prow.data(), &vbits);
  if (rc != GNNSTAGE_OK) return fail(nullptr, rc, "cannot pack row indices");

  Layout lay = make_layout(s, hp.f, hp.b, rank1);
  if (d->workspace_bytes < lay.total) {
    char buf[160];
    snprintf(buf, sizeof buf, "workspace too small: %zu bytes given, %zu needed", d->workspace_bytes, lay.total);
    return fail(nullptr, GNNSTAGE_ENOMEM, buf);
  }

  std::unique_ptr<gnnstage> holder(new gnnstage());  // freed on every early return, and when something below throws
  gnnstage *st = holder.get();
  st->s = s;
  st->lay = lay;
  st->vbits = vbits;
  st->alpha = d->alpha;
  if (s.res()) {
    for (int j = 0; j < s.L; ++j) {
      st->ln_g.push_back(static_cast<const float *>(d->ln_gamma[j]));
      st->ln_b.push_back(static_cast<const float *>(d->ln_beta[j]));
      st->d_ln_g.push_back(d->d_ln_gamma[j]);
      st->d_ln_b.push_back(d->d_ln_beta[j]);
    }
    st->ln_eps = d->ln_eps;
  }
  st->dropout_p = st->next_dropout_p = d->dropout_p;
  if (d->beta) st->beta.assign(d->beta, d->beta + s.L); else st->beta.assign(s.L, 0.f);
  st->W.assign(d->W, d->W + s.L);
  st->cur.assign(d->cur, d->cur + s.L + 1);
  st->hist.assign(d->hist, d->hist + s.L);
  st->dW.assign(d->dW, d->dW + s.L);
  if (d->bias) st->bias.assign(d->bias, d->bias + s.L); else st->bias.assign(s.L, nullptr);
  if (d->dbias) st->dbias.assign(d->dbias, d->dbias + s.L); else st->dbias.assign(s.L, nullptr);
  st->h0 = d->h0;
  st->grad_in = d->grad_in;
  st->grad_h0 = d->grad_h0;
  st->ws = static_cast<char *>(d->workspace);
  st->prof.init(s.L);
  st->n_classes = s.classes();
  st->h_row_ptr.assign(d->row_ptr, d->row_ptr + s.n + 1);
  if (hp.f.dense()) {  // the diagnostics walk the whole index, not the remainder
    st->h_pcol.resize((size_t)s.nnz);
    if (gnnstage_plan_pack(s.n, s.nnz, d->col_idx, s.K, s.chunk_ptr.data(), st->h_pcol.data(), &vbits) != GNNSTAGE_OK)
      return fail(nullptr, GNNSTAGE_EINVAL, "cannot pack column indices");
  } else {
    st->h_pcol = pcol;
  }

  // schedules: build on the host chunk by chunk, upload into the preallocated arrays
  const int classes = s.classes();
  auto build = [&](const HostDir &h, const uint32_t *packed, bool transposed, std::vector<TaskList> &lists) -> int {
    const int64_t *ptr = h.ptr;
    const int32_t *idx = h.idx;
    const PlanCounts &pc = h.pc;
    const int dir = transposed ? 1 : 0;
    lists.resize(s.K);
    int64_t t_off = 0, l_off = 0, s_off = 0;
    for (int c = 0; c < s.K; ++c) {
      TaskList &tl = lists[c];
      tl.slot_class = st->at<uint8_t>(transposed ? lay.b_slot_class : lay.f_slot_class) + s_off;
      s_off += pc.slots[c];
      tl.task_row = st->at<int32_t>(transposed ? lay.b_task_row : lay.f_task_row) + t_off;
      tl.task_e0 = st->at<int64_t>(transposed ? lay.b_task_e0 : lay.f_task_e0) + t_off;
      tl.task_ne = st->at<int32_t>(transposed ? lay.b_task_ne : lay.f_task_ne) + t_off;
      tl.task_slot = st->at<int32_t>(transposed ? lay.b_task_slot : lay.f_task_slot) + t_off;
      tl.lr_row = st->at<int32_t>(transposed ? lay.b_lr_row : lay.f_lr_row) + l_off;
      tl.lr_slot0 = st->at<int32_t>(transposed ? lay.b_lr_slot0 : lay.f_lr_slot0) + l_off;
      tl.lr_nslots = st->at<int32_t>(transposed ? lay.b_lr_n : lay.f_lr_n) + l_off;
      if (h.dense()) {
        tl.lr_dense0 = st->at<int32_t>(lay.d_lr_dense0[dir]) + l_off;
        tl.lr_ndense = st->at<int32_t>(lay.d_lr_ndense[dir]) + l_off;
        tl.lr_item0 = st->at<int32_t>(lay.d_lr_item0[dir]) + l_off;
        tl.item0 = h.chunk_item_off[(size_t)c];
        tl.n_items = (int)(h.chunk_item_off[(size_t)c + 1] - h.chunk_item_off[(size_t)c]);
      }
      t_off += pc.tasks[c];  // the arrays were sized from the upper bounds
      l_off += pc.longs[c];
      const int64_t cap = pc.tasks[c];
      if (cap == 0 && tl.n_items == 0) continue;
      std::vector<int32_t> row((size_t)std::max<int64_t>(cap, 1)), ne((size_t)std::max<int64_t>(cap, 1)), slot((size_t)std::max<int64_t>(cap, 1));
      std::vector<int64_t> e0((size_t)std::max<int64_t>(cap, 1));
      int64_t ns = 0;
      std::vector<int64_t> coff(classes + 1, 0);
      std::vector<uint8_t> sclass((size_t)std::max<int64_t>(pc.slots[c], 1), 255);
      // class bounds: equal shares of the chunk's entries over the id range, or (hotness classes) slices of
      // hot_rows ranks each, the ranks beyond the last slice belonging to no class
      std::vector<int64_t> cls_lo;
      if (h.hot.active) {
        cls_lo.resize((size_t)classes + 1);
        for (int q = 0; q <= classes; ++q) cls_lo[(size_t)q] = std::min<int64_t>((int64_t)q * s.hot_rows(), s.n);
      } else {
        cls_lo = class_bounds_by_entries(ptr, idx, s.n, s.chunk_ptr[c], s.chunk_ptr[c + 1], classes, s.chunk_ptr);
      }
      const int64_t got = gnnstage_plan_tasks(ptr, h.hot.active ? h.hot.rank.data() : idx, s.n, s.chunk_ptr[c], s.chunk_ptr[c + 1],
                                              pc.split[c], classes, cls_lo.data(), h.min_row, h.force_ptr(), cap, row.data(),
                                              e0.data(), ne.data(), slot.data(), &ns, coff.data(), sclass.data());
      if (got < 0 || got > cap || ns > pc.slots[c]) return GNNSTAGE_EINVAL;
      tl.n_classes = classes > 1 ? classes : 0;
      for (int q = 0; q <= tl.n_classes; ++q) tl.cls_off[q] = coff[q];
      tl.cls_chunk_entries.assign((size_t)tl.n_classes * s.K, 0);
      for (int q = 0; q < tl.n_classes; ++q)
        for (int64_t t = coff[q]; t < coff[q + 1]; ++t)
          for (int64_t e = e0[t]; e < e0[t] + ne[t]; ++e) tl.cls_chunk_entries[(size_t)q * s.K + (packed[e] >> vbits)] += 1;
      if (ns > 0 && hipMemcpy(tl.slot_class, sclass.data(), (size_t)ns, hipMemcpyHostToDevice) != hipSuccess)
        return GNNSTAGE_EHIP;
      tl.n_tasks = got;
      tl.n_slots = ns;
      // whole rows come last in the list: move the short ones behind the others (both parts keep their row order)
      const int short_row = s.short_row();
      if (short_row > 0) {
        int64_t first_whole = got;
        while (first_whole > 0 && slot[(size_t)first_whole - 1] < 0) --first_whole;
        std::vector<int64_t> ord;
        ord.reserve((size_t)(got - first_whole));
        for (int64_t t = first_whole; t < got; ++t)
          if (ne[(size_t)t] > short_row) ord.push_back(t);
        const int64_t n_other = (int64_t)ord.size();
        for (int64_t t = first_whole; t < got; ++t)
          if (ne[(size_t)t] <= short_row) ord.push_back(t);
        tl.n_short = (int64_t)ord.size() - n_other;
        if (tl.n_short > 0 && n_other > 0) {
          std::vector<int32_t> r2(ord.size()), n2(ord.size());
          std::vector<int64_t> e2(ord.size());
          for (size_t i = 0; i < ord.size(); ++i) {
            r2[i] = row[(size_t)ord[i]];
            n2[i] = ne[(size_t)ord[i]];
            e2[i] = e0[(size_t)ord[i]];
          }
          std::copy(r2.begin(), r2.end(), row.begin() + first_whole);
          std::copy(n2.begin(), n2.end(), ne.begin() + first_whole);
          std::copy(e2.begin(), e2.end(), e0.begin() + first_whole);
        }
      }
      // cut rows: their slots are consecutive, so sorting the pieces by slot groups them by row
      std::vector<std::pair<int32_t, int32_t>> sr;
      for (int64_t t = 0; t < got; ++t)
        if (slot[t] >= 0) sr.emplace_back(slot[t], row[t]);
      std::sort(sr.begin(), sr.end());
      std::vector<int32_t> lrow, lslot0, ln;
      for (const auto &p : sr) {
        if (lrow.empty() || lrow.back() != p.second) {
          lrow.push_back(p.second);
          lslot0.push_back(p.first);
          ln.push_back(0);
        }
        ln.back() += 1;
      }
      // rows of dense row blocks: their dense partial rows join the pieces (a row without any piece is added)
      std::vector<int32_t> ldense0(lrow.size(), 0), lndense(lrow.size(), 0), litem0(lrow.size(), 0);
      if (tl.n_items > 0) {
        std::vector<int32_t> where((size_t)(s.chunk_ptr[c + 1] - s.chunk_ptr[c]), -1);
        for (size_t i = 0; i < lrow.size(); ++i) where[(size_t)(lrow[i] - s.chunk_ptr[c])] = (int32_t)i;
        int64_t it = tl.item0;
        const int64_t it_end = tl.item0 + tl.n_items;
        while (it < it_end) {
          int64_t it2 = it;
          while (it2 < it_end && h.item_rb[(size_t)it2] == h.item_rb[(size_t)it]) ++it2;
          const int64_t p0 = (int64_t)h.item_rb[(size_t)it] * kDenseRB;
          const int64_t p1 = std::min<int64_t>(p0 + kDenseRB, s.chunk_ptr[c + 1] - s.chunk_ptr[c]);
          for (int64_t pp = p0; pp < p1; ++pp) {
            const int32_t r = h.dp.row_perm[(size_t)(s.chunk_ptr[c] + pp)];
            int32_t at = where[(size_t)(r - s.chunk_ptr[c])];
            if (at < 0) {
              at = (int32_t)lrow.size();
              lrow.push_back(r);
              lslot0.push_back(0);
              ln.push_back(0);
              ldense0.push_back(0);
              lndense.push_back(0);
              litem0.push_back(0);
            }
            ldense0[(size_t)at] = (int32_t)((it - tl.item0) * kDenseRB + (pp - p0));
            lndense[(size_t)at] = (int32_t)(it2 - it);
            litem0[(size_t)at] = (int32_t)(it - tl.item0);
          }
          it = it2;
        }
      }
      tl.n_long = (int64_t)lrow.size();
      if (tl.n_long > pc.longs[c]) return GNNSTAGE_EINVAL;
      if (h.dense() && tl.n_long > 0 &&
          (hipMemcpy(tl.lr_dense0, ldense0.data(), sizeof(int32_t) * tl.n_long, hipMemcpyHostToDevice) != hipSuccess ||
           hipMemcpy(tl.lr_ndense, lndense.data(), sizeof(int32_t) * tl.n_long, hipMemcpyHostToDevice) != hipSuccess ||
           hipMemcpy(tl.lr_item0, litem0.data(), sizeof(int32_t) * tl.n_long, hipMemcpyHostToDevice) != hipSuccess))
        return GNNSTAGE_EHIP;
      if (got > 0 &&
          (hipMemcpy(tl.task_row, row.data(), sizeof(int32_t) * got, hipMemcpyHostToDevice) != hipSuccess ||
           hipMemcpy(tl.task_e0, e0.data(), sizeof(int64_t) * got, hipMemcpyHostToDevice) != hipSuccess ||
           hipMemcpy(tl.task_ne, ne.data(), sizeof(int32_t) * got, hipMemcpyHostToDevice) != hipSuccess ||
           hipMemcpy(tl.task_slot, slot.data(), sizeof(int32_t) * got, hipMemcpyHostToDevice) != hipSuccess))
        return GNNSTAGE_EHIP;
      if (tl.n_long > 0 &&
          (hipMemcpy(tl.lr_row, lrow.data(), sizeof(int32_t) * tl.n_long, hipMemcpyHostToDevice) != hipSuccess ||
           hipMemcpy(tl.lr_slot0, lslot0.data(), sizeof(int32_t) * tl.n_long, hipMemcpyHostToDevice) != hipSuccess ||
           hipMemcpy(tl.lr_nslots, ln.data(), sizeof(int32_t) * tl.n_long, hipMemcpyHostToDevice) != hipSuccess))
        return GNNSTAGE_EHIP;
    }
    return GNNSTAGE_OK;
  };

  auto bail = [&](int code, const std::string &msg) { return fail(nullptr, code, msg); };
  if (hipMemcpy(st->at<int64_t>(lay.row_ptr), d->row_ptr, sizeof(int64_t) * (s.n + 1), hipMemcpyHostToDevice) != hipSuccess ||
      hipMemcpy(st->at<int64_t>(lay.t_ptr), t_ptr.data(), sizeof(int64_t) * (s.n + 1), hipMemcpyHostToDevice) != hipSuccess ||
      (hp.f.nnz > 0 && hipMemcpy(st->at<uint32_t>(lay.pcol), pcol.data(), sizeof(uint32_t) * hp.f.nnz, hipMemcpyHostToDevice) != hipSuccess) ||
      (hp.b.nnz > 0 && hipMemcpy(st->at<uint32_t>(lay.prow), prow.data(), sizeof(uint32_t) * hp.b.nnz, hipMemcpyHostToDevice) != hipSuccess))
    return bail(GNNSTAGE_EHIP, std::string("uploading the graph failed: ") + hipGetErrorString(hipGetLastError()));
  for (int dir = 0; dir < 2; ++dir) {  // dense plans
    const HostDir &h = dir ? hp.b : hp.f;
    if (!h.dense()) continue;
    const DensePlan &dp = h.dp;
    const size_t nb = (size_t)dp.n_blocks(), ne = dp.ent_pos.size(), ni = h.item_rb.size();  // ne: real entries, without padding
    std::vector<uint32_t> colslot(dp.colslot_vertex.size());
    std::vector<int32_t> chunk_of((size_t)s.n);
    for (int c = 0; c < s.K; ++c)
      for (int64_t v = s.chunk_ptr[c]; v < s.chunk_ptr[c + 1]; ++v) chunk_of[(size_t)v] = c;
    for (size_t i = 0; i < colslot.size(); ++i) {
      const int32_t v = dp.colslot_vertex[i];
      colslot[i] = v < 0 ? 0xffffffffu : ((uint32_t)v | ((uint32_t)chunk_of[(size_t)v] << vbits));
    }
    if (hipMemcpy(st->at<int64_t>(lay.rem_ptr[dir]), dp.rem_ptr.data(), sizeof(int64_t) * (s.n + 1), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(st->at<int32_t>(lay.d_blk_cb[dir]), dp.blk_cb.data(), sizeof(int32_t) * nb, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(st->at<uint32_t>(lay.d_colslot[dir]), colslot.data(), sizeof(uint32_t) * colslot.size(), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(st->at<int32_t>(lay.d_item_rb[dir]), h.item_rb.data(), sizeof(int32_t) * ni, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(st->at<int64_t>(lay.d_item_b0[dir]), h.item_b0.data(), sizeof(int64_t) * ni, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(st->at<int32_t>(lay.d_item_nb[dir]), h.item_nb.data(), sizeof(int32_t) * ni, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(st->at<ChunkMask>(lay.d_item_chunks[dir]), h.item_chunks.data(), sizeof(ChunkMask) * ni, hipMemcpyHostToDevice) != hipSuccess)
      return bail(GNNSTAGE_EHIP, std::string("uploading the dense blocks failed: ") + hipGetErrorString(hipGetLastError()));
    if (rank1) {
      // patterns and the two scale vectors.  GCN normalisation: s_row = s_col = 1 / sqrt(row length in A + I).
      // Mean aggregator: 1 / |N(v)| belongs to the destination v, which is the row of a forward block and the
      // column of a block of the transposed index.
      auto row_len = [&](int64_t v) { return d->row_ptr[v + 1] - d->row_ptr[v]; };
      auto inv_sqrt = [&](int64_t v) { return (float)(1.0 / sqrt((double)row_len(v))); };
      auto inv_len = [&](int64_t v) { return row_len(v) > 0 ? 1.f / (float)row_len(v) : 0.f; };
      auto row_scale = [&](int64_t v) { return !s.sage() ? inv_sqrt(v) : dir == 0 ? inv_len(v) : 1.f; };
      auto col_scale = [&](int64_t v) { return !s.sage() ? inv_sqrt(v) : dir == 0 ? 1.f : inv_len(v); };
      std::vector<uint32_t> bits(nb * 256, 0u);
      for (size_t b = 0; b < nb; ++b)
        for (int64_t e = dp.blk_e0[b]; e < dp.blk_e0[b + 1]; ++e) {
          const uint32_t pos = dp.ent_pos[(size_t)e], r = pos >> 8, c = pos & 255u;
          bits[b * 256 + r * 2 + (c >> 5)] |= 1u << (c & 31u);
        }
      std::vector<float> colscale(colslot.size(), 0.f), rowscale((size_t)h.rowscale_off.back(), 0.f);
      for (size_t i = 0; i < colslot.size(); ++i)
        if (dp.colslot_vertex[i] >= 0) colscale[i] = col_scale(dp.colslot_vertex[i]);
      for (int k = 0; k < s.K; ++k)
        for (int64_t pp = 0; pp < s.chunk_ptr[k + 1] - s.chunk_ptr[k]; ++pp)
          rowscale[(size_t)(h.rowscale_off[(size_t)k] + pp)] = row_scale(dp.row_perm[(size_t)(s.chunk_ptr[k] + pp)]);
      if (hipMemcpy(st->at<uint32_t>(lay.d_bits[dir]), bits.data(), sizeof(uint32_t) * bits.size(), hipMemcpyHostToDevice) != hipSuccess ||
          hipMemcpy(st->at<float>(lay.d_colscale[dir]), colscale.data(), sizeof(float) * colscale.size(), hipMemcpyHostToDevice) != hipSuccess ||
          hipMemcpy(st->at<float>(lay.d_rowscale[dir]), rowscale.data(), sizeof(float) * rowscale.size(), hipMemcpyHostToDevice) != hipSuccess)
        return bail(GNNSTAGE_EHIP, "uploading the dense patterns failed");
      st->rowscale_off[dir] = h.rowscale_off;
    } else {
      const size_t ne_pad = (size_t)h.padded_entries();
      std::vector<uint32_t> ent_w(ne_pad, 0u);
      std::vector<uint16_t> ent_pos(ne_pad, (uint16_t)0xffff);
      std::vector<int64_t> blk_e0(nb + 1, 0);
      for (int k = 0; k < s.K; ++k)
        for (int64_t b = dp.chunk_blk_off[(size_t)k]; b < dp.chunk_blk_off[(size_t)k + 1]; ++b) {
          int64_t at = blk_e0[(size_t)b];
          for (int64_t e = dp.blk_e0[(size_t)b]; e < dp.blk_e0[(size_t)b + 1]; ++e, ++at) {
            const uint32_t pos = dp.ent_pos[(size_t)e];
            const int64_t e_csr = dir ? t_edge[(size_t)dp.ent_orig[(size_t)e]] : dp.ent_orig[(size_t)e];
            const float wgt = d->edge_val[e_csr];
            const uint16_t hi = bf16_bits_rne(wgt), lo = bf16_bits_rne(wgt - bf16_bits_to_f32(hi));
            ent_w[(size_t)at] = (uint32_t)hi | ((uint32_t)lo << 16);
            ent_pos[(size_t)at] = (uint16_t)pos;
          }
          blk_e0[(size_t)b + 1] = (at + 7) / 8 * 8;
        }
      if (hipMemcpy(st->at<int64_t>(lay.d_blk_e0[dir]), blk_e0.data(), sizeof(int64_t) * (nb + 1), hipMemcpyHostToDevice) != hipSuccess ||
          hipMemcpy(st->at<uint16_t>(lay.d_ent_pos[dir]), ent_pos.data(), sizeof(uint16_t) * ne_pad, hipMemcpyHostToDevice) != hipSuccess ||
          hipMemcpy(st->at<uint32_t>(lay.d_ent_w[dir]), ent_w.data(), sizeof(uint32_t) * ne_pad, hipMemcpyHostToDevice) != hipSuccess)
        return bail(GNNSTAGE_EHIP, "uploading the dense entries failed");
      if (launch_fill_zero(st->at<char>(lay.d_tiles[dir]), sizeof(uint16_t) * nb * 2 * kDenseRB * kDenseCB, nullptr) != 0 ||
          launch_dense_expand(st->at<int64_t>(lay.d_blk_e0[dir]), st->at<uint16_t>(lay.d_ent_pos[dir]),
                              st->at<uint32_t>(lay.d_ent_w[dir]), st->at<char>(lay.d_tiles[dir]), (int64_t)nb, nullptr) != 0)
        return bail(GNNSTAGE_EHIP, "expanding the dense blocks failed");
    }
    st->dense_rank1 = rank1;
    if (launch_fill_zero(st->at<char>(lay.zero_row), 512, nullptr) != 0) return bail(GNNSTAGE_EHIP, "clearing the zero row failed");
    st->dense_on[dir] = true;
    st->dense_entries[dir] = (int64_t)ne;
  }
  if (d->edge_val) {
    std::vector<float> fval, tval((size_t)hp.b.nnz);
    const float *fv = d->edge_val;
    // entry i of the index a direction's sparse kernels see -> its position in that direction's full index:
    // through the hotness order (if any), then through the dense plan's remainder (if any)
    auto full_pos = [](const HostDir &h, int64_t i) {
      if (h.hot.active) i = h.hot.orig[(size_t)i];
      return h.dense() ? h.dp.rem_orig[(size_t)i] : i;
    };
    if (hp.f.dense() || hp.f.hot.active) {
      fval.resize((size_t)hp.f.nnz);
      for (int64_t i = 0; i < hp.f.nnz; ++i) fval[(size_t)i] = d->edge_val[full_pos(hp.f, i)];
      fv = fval.data();
    }
    for (int64_t i = 0; i < hp.b.nnz; ++i) tval[(size_t)i] = d->edge_val[t_edge[(size_t)full_pos(hp.b, i)]];
    if ((hp.f.nnz > 0 && hipMemcpy(st->at<float>(lay.val), fv, sizeof(float) * hp.f.nnz, hipMemcpyHostToDevice) != hipSuccess) ||
        (hp.b.nnz > 0 && hipMemcpy(st->at<float>(lay.tval), tval.data(), sizeof(float) * hp.b.nnz, hipMemcpyHostToDevice) != hipSuccess))
      return bail(GNNSTAGE_EHIP, "uploading edge values failed");
  } else {
    // Section 2.1 weights from the row lengths of A + I, for the (remaining) CSR entries and for their transposed copies
    const int64_t *rp = st->at<int64_t>(lay.row_ptr);
    const int64_t *fp = hp.f.dense() ? st->at<int64_t>(lay.rem_ptr[0]) : rp;
    const int64_t *bp = hp.b.dense() ? st->at<int64_t>(lay.rem_ptr[1]) : st->at<int64_t>(lay.t_ptr);
    if (launch_gcn_norm(fp, st->at<uint32_t>(lay.pcol), vbits, rp, s.n, st->at<float>(lay.val), nullptr) != 0 ||
        launch_gcn_norm(bp, st->at<uint32_t>(lay.prow), vbits, rp, s.n, st->at<float>(lay.tval), nullptr) != 0)
      return bail(GNNSTAGE_EHIP, "normalisation kernel launch failed");
  }
  rc = build(hp.f, pcol.data(), false, st->ftasks);
  if (rc == GNNSTAGE_OK) rc = build(hp.b, prow.data(), true, st->btasks);
  if (rc != GNNSTAGE_OK) return bail(rc, "building the launch schedule failed");
  if (hipDeviceSynchronize() != hipSuccess) return bail(GNNSTAGE_EHIP, "device synchronisation failed after create");
  *out = holder.release();
  return GNNSTAGE_OK;
}
GNNSTAGE_GUARD_INT

extern "C" int gnnstage_destroy(gnnstage_t *st) try {
  if (!st) return GNNSTAGE_EINVAL;
  const hipError_t e = hipDeviceSynchronize();
  st->prof.destroy();
  delete st;
  return e == hipSuccess ? GNNSTAGE_OK : GNNSTAGE_EHIP;
}
GNNSTAGE_GUARD_INT

extern "C" int stage_forward_chunk(gnnstage_t *st, int32_t k, int32_t pos, void *hip_stream) try {
  if (!st) return GNNSTAGE_EINVAL;
  const Shape &s = st->s;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (k < 0 || k >= s.K) return fail(st, GNNSTAGE_ERANGE, "chunk id out of range");
  const int cd = st->cdtype();
  const size_t celt = s.elt();
  if (pos == 0) {  // a new pass: V_processed <- empty
    st->order.clear();
    st->fmask = ChunkMask{};
    st->bmask = ChunkMask{};
    st->n_bwd = 0;
    st->wgrad_pending.assign((size_t)s.K, 0);  // what an abandoned backward pass still owed is dropped with it
    st->dropout_p = st->next_dropout_p;
    st->dropout_seed = st->next_dropout_seed;
    {
      Timed t(st, stream, 6);
      for (int j = 0; j < s.L; ++j) {
        // GraphSage: W[j] = [W_self ; W_neigh]; Wt / Wn take the half that multiplies the aggregation
        const char *Wagg = static_cast<const char *>(st->W[j]) + (s.sage() ? s.w_half(j) * s.elt() : 0);
        HIP_TRY(st, launch_stage_weights(Wagg, cd, s.dims[j], s.dims[j + 1], st->at<char>(st->lay.Wt[j]), s.ld[j],
                                         st->at<char>(st->lay.Wn[j]), s.ld[j + 1], stream));
        if (s.sage())
          HIP_TRY(st, launch_stage_weights(st->W[j], cd, s.dims[j], s.dims[j + 1], st->at<char>(st->lay.Wt_self[j]), s.ld[j],
                                           st->at<char>(st->lay.Wn_self[j]), s.ld[j + 1], stream));
      }
    }
    if (s.res()) {
      const int rc = res_pass_start(st, stream);
      if (rc != GNNSTAGE_OK) return rc;
    }
    // transform-first layers: the historical rows are constants of the pass, transform them once
    for (int j = 0; j < s.L; ++j) {
      if (!s.tf[j]) continue;
      Timed t(st, stream, 1, j);
      GemmNtArgs g{};
      g.ws_min_rows = st->s.tune.gemm_ws_min_rows;
      g.A = st->hist[j];
      g.a_dtype = st->level_dtype(j);
      g.lda = s.dims[j];
      g.Bt = st->at<char>(st->lay.Wt[j]);
      g.ldb = s.ld[j];
      g.M = (int)s.n;
      g.N = s.dims[j + 1];
      g.K = s.dims[j];
      g.Kp = s.ld[j];
      g.epilogue = EPI_PLAIN;
      g.out = st->at<char>(st->lay.Th[j]);
      g.out_dtype = cd;
      g.out_ld = s.ld[j + 1];
      HIP_TRY(st, launch_gemm_nt(g, cd, stream));
    }
  }
  if (pos != (int32_t)st->order.size()) return fail(st, GNNSTAGE_EORDER, "pos_in_pass does not continue the current pass");
  if (mask_test(st->fmask, (uint32_t)k)) return fail(st, GNNSTAGE_EORDER, "chunk already processed in this pass");
  st->order.push_back(k);
  mask_set(st->fmask, k);  // C_k joins V_processed before its layers run
  if ((int)st->order.size() == s.K) st->cur_stale = false;  // after this call every current row is of this pass

  const int64_t row0 = s.chunk_ptr[k], M = s.chunk_ptr[k + 1] - row0;
  if (M == 0) return GNNSTAGE_OK;
  if (s.res()) return res_forward_chunk(st, k, stream);
  for (int j = 0; j < s.L; ++j) {
    if (s.tf[j]) {
      // transform the chunk's current rows, then aggregate transformed rows (current or historical)
      const bool shared = st->hist[j] == st->cur[j];  // level never changes: one transformed table serves both
      char *Th = st->at<char>(st->lay.Th[j]);
      char *Tc = shared ? Th : st->at<char>(st->lay.Tc[j]);
      if (!shared) {
        Timed t(st, stream, 1, j);
        GemmNtArgs g{};
        g.ws_min_rows = st->s.tune.gemm_ws_min_rows;
        g.A = static_cast<const char *>(st->cur[j]) + (size_t)row0 * s.dims[j] * st->level_elt(j);
        g.a_dtype = st->level_dtype(j);
        g.lda = s.dims[j];
        g.Bt = st->at<char>(st->lay.Wt[j]);
        g.ldb = s.ld[j];
        g.M = (int)M;
        g.N = s.dims[j + 1];
        g.K = s.dims[j];
        g.Kp = s.ld[j];
        g.epilogue = EPI_PLAIN;
        g.out = Tc + (size_t)row0 * s.ld[j + 1] * celt;
        g.out_dtype = cd;
        g.out_ld = s.ld[j + 1];
        HIP_TRY(st, launch_gemm_nt(g, cd, stream));
      }
      SpmmArgs a = base_spmm(st, false, k);
      a.src_sel = Tc;
      a.src_unsel = Th;
      a.d = s.dims[j + 1];
      a.src_ld = s.ld[j + 1];
      a.out = st->cur[j + 1];
      a.out_ld = s.dims[j + 1];
      a.out_row0 = 0;
      a.epilogue = SPMM_BIAS_RELU;
      a.bias = static_cast<const float *>(st->bias[j]);
      HIP_TRY(st, run_spmm(st, a, false, k, cd, cd, stream, 0, j));
      if (st->output_dropout())  // on the rows just written, in place
        HIP_TRY(st, launch_dropout_rows(static_cast<char *>(st->cur[j + 1]) + (size_t)row0 * s.dims[j + 1] * celt, cd, M, s.dims[j + 1],
                                        s.dims[j + 1], st->dropout(j, row0), stream));
      continue;
    }
    char *Zj = st->at<char>(st->lay.Z[j]);
    {
      SpmmArgs a = base_spmm(st, false, k);
      a.src_sel = st->cur[j];
      a.src_unsel = st->hist[j];
      a.d = s.dims[j];
      a.src_ld = s.dims[j];
      a.out = Zj;
      a.out_ld = s.ld[j];
      a.out_row0 = 0;
      if (s.variant == GNNSTAGE_GCNII) {
        a.epilogue = SPMM_MIX;
        a.aux = st->h0;
        a.aux_ld = s.dims[j];
        a.s_acc = 1.f - st->alpha;
        a.s_aux = st->alpha;
      } else {
        a.epilogue = SPMM_PLAIN;
      }
      HIP_TRY(st, run_spmm(st, a, false, k, st->level_dtype(j), cd, stream, 0, j));
    }
    if (s.sage()) {  // the vertex's own row through W_self, kept in fp32 until the layer's epilogue adds it
      Timed t(st, stream, 1, j);
      GemmNtArgs g{};
      g.ws_min_rows = st->s.tune.gemm_ws_min_rows;
      g.A = static_cast<const char *>(st->cur[j]) + (size_t)row0 * s.dims[j] * st->level_elt(j);
      g.a_dtype = st->level_dtype(j);
      g.lda = s.dims[j];
      g.Bt = st->at<char>(st->lay.Wt_self[j]);
      g.ldb = s.ld[j];
      g.M = (int)M;
      g.N = s.dims[j + 1];
      g.K = s.dims[j];
      g.Kp = s.ld[j];
      g.epilogue = EPI_PLAIN;
      g.out = st->at<float>(st->lay.self_fwd);
      g.out_dtype = DT_F32;
      g.out_ld = s.ld[j + 1];
      HIP_TRY(st, launch_gemm_nt(g, cd, stream));
    }
    {
      Timed t(st, stream, 1, j);
      GemmNtArgs g{};
      g.ws_min_rows = st->s.tune.gemm_ws_min_rows;
      g.A = Zj + (size_t)row0 * s.ld[j] * celt;
      g.a_dtype = cd;
      g.lda = s.ld[j];
      g.Bt = st->at<char>(st->lay.Wt[j]);
      g.ldb = s.ld[j];
      g.M = (int)M;
      g.N = s.dims[j + 1];
      g.K = s.dims[j];
      g.Kp = s.ld[j];
      if (s.variant == GNNSTAGE_GCNII) {
        g.epilogue = EPI_FWD_GCNII;
        g.aux = g.A;
        g.aux_dtype = cd;
        g.aux_ld = s.ld[j];
        g.beta = st->beta[j];
      } else {
        g.epilogue = EPI_FWD_GCN;
        g.bias = static_cast<const float *>(st->bias[j]);
        if (s.sage()) {
          g.epilogue = EPI_FWD_ADD;
          g.aux = st->at<float>(st->lay.self_fwd);
          g.aux_dtype = DT_F32;
          g.aux_ld = s.ld[j + 1];
        }
      }
      g.out = static_cast<char *>(st->cur[j + 1]) + (size_t)row0 * s.dims[j + 1] * celt;
      g.out_dtype = cd;
      g.out_ld = s.dims[j + 1];
      HIP_TRY(st, launch_gemm_nt(g, cd, stream));
      if (st->output_dropout())  // on the rows just written, in place
        HIP_TRY(st, launch_dropout_rows(g.out, cd, M, s.dims[j + 1], s.dims[j + 1], st->dropout(j, row0), stream));
    }
  }
  return GNNSTAGE_OK;
}
GNNSTAGE_GUARD_INT

namespace {
// Weight (and bias) gradients of the aggregate-first layers that the backward calls made so far still owe:
// dW_j += scale * Z_j^T dY_j over the rows of every maximal run of chunks whose backward call has run.  A complete
// pass is one run, i.e. one product per layer over all n rows.
int flush_deferred_wgrad(gnnstage *st, hipStream_t stream) {
  const Shape &s = st->s;
  if (!s.defer_wgrad() || st->wgrad_pending.empty()) return GNNSTAGE_OK;
  const int cd = st->cdtype();
  const size_t celt = s.elt();
  float *gemm_partial = st->at<float>(st->lay.gemm_partial);
  float *bias_partial = st->at<float>(st->lay.bias_partial);
  int c = 0;
  while (c < s.K) {
    if (!st->wgrad_pending[(size_t)c]) {
      ++c;
      continue;
    }
    int c1 = c;
    while (c1 < s.K && st->wgrad_pending[(size_t)c1]) st->wgrad_pending[(size_t)c1++] = 0;
    const int64_t r0 = s.chunk_ptr[c], M = s.chunk_ptr[c1] - r0;
    c = c1;
    if (M <= 0) continue;
    if (M > 0x7fffffff) return fail(st, GNNSTAGE_ENOTSUP, "more than 2^31 - 1 rows in one weight-gradient product");
    for (int j = s.L - 1; j >= 0; --j) {
      if (s.tf[j]) continue;  // transform-first layers: finish_transform_first
      const char *dY = st->at<char>(st->lay.dY[j]) + (size_t)r0 * s.ld[j + 1] * celt;
      const bool fuse_bias = s.has_bias() && cd == DT_BF16;
      Timed t(st, stream, 4, j);
      if (s.has_bias() && !fuse_bias)
        HIP_TRY(st, launch_colsum_add(dY, cd, s.ld[j + 1], (int)M, s.dims[j + 1], bias_partial, kMaxSplits, st->dbias[j], stream));
      GemmTnArgs w{};
      w.wide_min_rows = st->s.tune.gemm_wide_min_rows;
      w.A = st->at<char>(st->lay.Z[j]) + (size_t)r0 * s.ld[j] * celt;
      w.a_dtype = cd;
      w.lda = s.ld[j];
      w.B = dY;
      w.ldb = s.ld[j + 1];
      w.M = (int)M;
      w.I = s.dims[j];
      w.O = s.dims[j + 1];
      w.scale = s.variant == GNNSTAGE_GCNII ? st->beta[j] : 1.f;
      w.dW = st->dW[j] + (s.sage() ? s.w_half(j) : 0);  // GraphSage: W_neigh is the lower half
      w.partial = gemm_partial;
      w.max_splits = kMaxSplits;
      if (fuse_bias) {
        w.dbias = st->dbias[j];
        w.bias_partial = bias_partial;
      }
      HIP_TRY(st, launch_gemm_tn(w, cd, stream));
      if (s.sage()) {  // dW_self += h_v^T dY over the rows' own (current) level-j values
        GemmTnArgs ws{};
        ws.wide_min_rows = st->s.tune.gemm_wide_min_rows;
        ws.A = static_cast<const char *>(st->cur[j]) + (size_t)r0 * s.dims[j] * st->level_elt(j);
        ws.a_dtype = st->level_dtype(j);
        ws.lda = s.dims[j];
        ws.B = dY;
        ws.ldb = s.ld[j + 1];
        ws.M = (int)M;
        ws.I = s.dims[j];
        ws.O = s.dims[j + 1];
        ws.scale = 1.f;
        ws.dW = st->dW[j];
        ws.partial = gemm_partial;
        ws.max_splits = kMaxSplits;
        HIP_TRY(st, launch_gemm_tn(ws, cd, stream));
      }
    }
  }
  return GNNSTAGE_OK;
}
}  // namespace

extern "C" int gnnstage_flush_weight_gradients(gnnstage_t *st, void *hip_stream) try {
  if (!st) return GNNSTAGE_EINVAL;
  return flush_deferred_wgrad(st, static_cast<hipStream_t>(hip_stream));
}
GNNSTAGE_GUARD_INT

extern "C" int stage_backward_chunk(gnnstage_t *st, int32_t k, const void *grad_out_rows, void *hip_stream) try {
  if (!st) return GNNSTAGE_EINVAL;
  const Shape &s = st->s;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (k < 0 || k >= s.K) return fail(st, GNNSTAGE_ERANGE, "chunk id out of range");
  if ((int)st->order.size() != s.K) return fail(st, GNNSTAGE_EORDER, "backward before the forward pass covered every chunk");
  if (st->n_bwd >= s.K) return fail(st, GNNSTAGE_EORDER, "backward pass already complete");
  if (st->order[s.K - 1 - st->n_bwd] != k) return fail(st, GNNSTAGE_EORDER, "backward must walk the chunks in reverse forward order");
  const int64_t row0 = s.chunk_ptr[k], M = s.chunk_ptr[k + 1] - row0;
  if (M > 0 && !grad_out_rows) return fail(st, GNNSTAGE_EINVAL, "grad_out_rows is NULL");
  st->n_bwd += 1;
  mask_set(st->bmask, k);
  if (s.res()) return res_backward_chunk(st, k, grad_out_rows, stream);
  // what the last call of a pass owes beyond its own rows: the deferred weight-gradient products, then the
  // history-side weight gradient of the transform-first layers
  auto end_of_pass = [&]() -> int {
    if (st->n_bwd != s.K) return GNNSTAGE_OK;
    const int rc = flush_deferred_wgrad(st, stream);
    return rc != GNNSTAGE_OK ? rc : finish_transform_first(st, stream);
  };
  // an empty chunk has no rows of its own, but the end-of-pass work still runs when it is the last call of the pass
  if (M == 0) return end_of_pass();

  const int cd = st->cdtype();
  const size_t celt = s.elt();
  const bool defer = s.defer_wgrad();
  char *G[2] = {st->at<char>(st->lay.G[0]), st->at<char>(st->lay.G[1])};
  float *gemm_partial = st->at<float>(st->lay.gemm_partial);
  float *bias_partial = st->at<float>(st->lay.bias_partial);
  // Where dY_j = dL/d(pre-activation of layer j) of the chunk's rows lives, [M x ld_{j+1}], zero in the padding
  // columns.  With deferred weight gradients: the chunk's rows of a matrix over all n rows (transform-first layers
  // keep that matrix anyway, it is what later chunks' transposed aggregations gather); otherwise one of two
  // chunk-sized scratch matrices, used alternately.
  int gi = 0;
  auto full_dY = [&](int j) { return st->at<char>(s.tf[j] ? st->lay.dZ[j] : st->lay.dY[j]); };
  auto dY_rows = [&](int j) -> char * { return defer ? full_dY(j) + (size_t)row0 * s.ld[j + 1] * celt : G[gi]; };
  if (defer) st->wgrad_pending[(size_t)k] = 1;
  {
    Timed t(st, stream, 6);
    const char *top = static_cast<const char *>(st->cur[s.L]) + (size_t)row0 * s.dims[s.L] * celt;
    HIP_TRY(st, launch_relu_mask(grad_out_rows, top, cd, M, s.dims[s.L], dY_rows(s.L - 1), s.ld[s.L], st->mask_scale(), stream));
  }
  for (int j = s.L - 1; j >= 0; --j) {
    const char *dY = dY_rows(j);
    // bias gradient = column sums of dY: fused into the weight-gradient product where that product reads dY
    // (aggregate-first layers of the bf16 stage), a kernel of its own otherwise; aggregate-first layers with
    // deferred weight gradients take it with the deferred product
    const bool fuse_bias = s.has_bias() && !s.tf[j] && cd == DT_BF16;
    if (s.has_bias() && !fuse_bias && !(defer && !s.tf[j])) {
      Timed t(st, stream, 4, j);
      HIP_TRY(st, launch_colsum_add(dY, cd, s.ld[j + 1], (int)M, s.dims[j + 1], bias_partial, kMaxSplits, st->dbias[j], stream));
    }
    const bool need_prev = j > 0 || s.need_input_grad;
    if (s.tf[j]) {
      // Layer computed as A_hat (H W).  With T = H W:  dL/dW = cur^T dT_cur + hist^T dT_hist, where
      // dT_cur[u] sums A_vu dY[v] over the readers v that saw u's CURRENT row (exactly the vertices
      // already processed in this backward pass) and dT_hist over the readers that saw its history.
      // dT_cur + dT_hist is the unmasked transposed aggregation, known only when every chunk's dY is:
      //   dW += (cur - hist)[C_k]^T dT_cur[C_k]   here, per chunk,
      //   dW += hist^T (A_hat^T dY)                after the last chunk (finish_transform_first).
      const bool shared = st->hist[j] == st->cur[j];
      char *dYfull = st->at<char>(st->lay.dZ[j]);
      if (!defer) {
        Timed t(st, stream, 6);
        HIP_TRY(st, launch_copy(dY, dYfull + (size_t)row0 * s.ld[j + 1] * celt, (size_t)M * s.ld[j + 1] * celt, stream));
      }
      if (shared && !need_prev) continue;  // nothing else depends on dT_cur
      char *dT = defer ? G[0] : G[gi ^ 1];
      {
        SpmmArgs a = base_spmm(st, true, k);
        a.src_sel = dYfull;
        a.src_unsel = nullptr;  // Section 3.4: nothing flows back from unprocessed vertices
        a.d = s.dims[j + 1];
        a.src_ld = s.ld[j + 1];
        a.out = dT;
        a.out_ld = s.ld[j + 1];
        a.out_row0 = row0;
        a.epilogue = SPMM_PLAIN;
        HIP_TRY(st, run_spmm(st, a, true, k, cd, cd, stream, 2, j));
      }
      if (!shared) {
        Timed t(st, stream, 4, j);
        GemmTnArgs w{};
        w.wide_min_rows = st->s.tune.gemm_wide_min_rows;
        w.a_dtype = st->level_dtype(j);
        w.lda = s.dims[j];
        w.B = dT;
        w.ldb = s.ld[j + 1];
        w.M = (int)M;
        w.I = s.dims[j];
        w.O = s.dims[j + 1];
        w.dW = st->dW[j];
        w.partial = gemm_partial;
        w.max_splits = kMaxSplits;
        w.A = static_cast<const char *>(st->cur[j]) + (size_t)row0 * s.dims[j] * st->level_elt(j);
        w.scale = 1.f;
        HIP_TRY(st, launch_gemm_tn(w, cd, stream));
        w.A = static_cast<const char *>(st->hist[j]) + (size_t)row0 * s.dims[j] * st->level_elt(j);
        w.scale = -1.f;
        HIP_TRY(st, launch_gemm_tn(w, cd, stream));
      }
      if (!need_prev) continue;
      {
        Timed t(st, stream, 3, j);
        GemmNtArgs g{};
        g.ws_min_rows = st->s.tune.gemm_ws_min_rows;
        g.A = dT;
        g.a_dtype = cd;
        g.lda = s.ld[j + 1];
        g.Bt = st->at<char>(st->lay.Wn[j]);
        g.ldb = s.ld[j + 1];
        g.M = (int)M;
        g.N = s.dims[j];
        g.K = s.dims[j + 1];
        g.Kp = s.ld[j + 1];
        if (j > 0) {
          g.epilogue = EPI_MASK;
          g.mask_scale = st->mask_scale();
          g.aux = static_cast<const char *>(st->cur[j]) + (size_t)row0 * s.dims[j] * celt;
          g.aux_dtype = cd;
          g.aux_ld = s.dims[j];
          g.out = defer ? dY_rows(j - 1) : G[gi];  // without deferral dY_j is dead by now and its scratch is reused
          g.out_dtype = cd;
          g.out_ld = s.ld[j];
          g.out_pad = s.ld[j];
        } else {
          g.epilogue = EPI_PLAIN;
          g.out = static_cast<char *>(st->grad_in) + (size_t)row0 * s.dims[0] * st->level_elt(0);
          g.out_dtype = st->level_dtype(0);
          g.out_ld = s.dims[0];
        }
        HIP_TRY(st, launch_gemm_nt(g, cd, stream));
      }
      continue;  // without deferral the next dY sits in G[gi] again
    }
    if (!defer) {
      const char *Zrows = st->at<char>(st->lay.Z[j]) + (size_t)row0 * s.ld[j] * celt;
      Timed t(st, stream, 4, j);
      GemmTnArgs w{};
      w.wide_min_rows = st->s.tune.gemm_wide_min_rows;
      w.A = Zrows;
      w.a_dtype = cd;
      w.lda = s.ld[j];
      w.B = dY;
      w.ldb = s.ld[j + 1];
      w.M = (int)M;
      w.I = s.dims[j];
      w.O = s.dims[j + 1];
      w.scale = s.variant == GNNSTAGE_GCNII ? st->beta[j] : 1.f;
      w.dW = st->dW[j] + (s.sage() ? s.w_half(j) : 0);  // GraphSage: W_neigh is the lower half
      w.partial = gemm_partial;
      w.max_splits = kMaxSplits;
      if (fuse_bias) {
        w.dbias = st->dbias[j];
        w.bias_partial = bias_partial;
      }
      HIP_TRY(st, launch_gemm_tn(w, cd, stream));
      if (s.sage()) {  // dW_self += h_v^T dY over the chunk's own (current) rows
        GemmTnArgs ws{};
        ws.wide_min_rows = st->s.tune.gemm_wide_min_rows;
        ws.A = static_cast<const char *>(st->cur[j]) + (size_t)row0 * s.dims[j] * st->level_elt(j);
        ws.a_dtype = st->level_dtype(j);
        ws.lda = s.dims[j];
        ws.B = dY;
        ws.ldb = s.ld[j + 1];
        ws.M = (int)M;
        ws.I = s.dims[j];
        ws.O = s.dims[j + 1];
        ws.scale = 1.f;
        ws.dW = st->dW[j];
        ws.partial = gemm_partial;
        ws.max_splits = kMaxSplits;
        HIP_TRY(st, launch_gemm_tn(ws, cd, stream));
      }
    }
    if (!need_prev) break;
    char *dZj = st->at<char>(st->lay.dZ[j]);
    {
      Timed t(st, stream, 3, j);
      GemmNtArgs g{};
      g.ws_min_rows = st->s.tune.gemm_ws_min_rows;
      g.A = dY;
      g.a_dtype = cd;
      g.lda = s.ld[j + 1];
      g.Bt = st->at<char>(st->lay.Wn[j]);
      g.ldb = s.ld[j + 1];
      g.M = (int)M;
      g.N = s.dims[j];
      g.K = s.dims[j + 1];
      g.Kp = s.ld[j + 1];
      if (s.variant == GNNSTAGE_GCNII) {
        g.epilogue = EPI_DGRAD_GCNII;
        g.aux = dY;
        g.aux_dtype = cd;
        g.aux_ld = s.ld[j + 1];
        g.alpha = st->alpha;
        g.beta = st->beta[j];
        g.h0grad = st->grad_h0 ? st->grad_h0 + (size_t)row0 * s.dims[j] : nullptr;
        g.h0_ld = s.dims[j];
      } else {
        g.epilogue = EPI_PLAIN;
      }
      g.out = dZj + (size_t)row0 * s.ld[j] * celt;
      g.out_dtype = cd;
      g.out_ld = s.ld[j];
      HIP_TRY(st, launch_gemm_nt(g, cd, stream));
      if (s.sage()) {  // the gradient that reaches the chunk's own rows directly: dY W_self^T
        g.Bt = st->at<char>(st->lay.Wn_self[j]);
        g.out = st->at<char>(st->lay.self_bwd);
        HIP_TRY(st, launch_gemm_nt(g, cd, stream));
      }
    }
    {
      SpmmArgs a = base_spmm(st, true, k);
      a.src_sel = dZj;
      a.src_unsel = nullptr;  // Section 3.4: nothing flows back from unprocessed vertices
      a.d = s.dims[j];
      a.src_ld = s.ld[j];
      if (s.sage()) {
        a.add = st->at<char>(st->lay.self_bwd);
        a.add_ld = s.ld[j];
        a.add_row0 = row0;
      }
      if (j > 0) {
        if (defer) {  // straight into the chunk's rows of dY_{j-1}
          a.out = full_dY(j - 1);
          a.out_row0 = 0;
        } else {
          a.out = G[gi ^ 1];
          a.out_row0 = row0;
        }
        a.out_ld = s.ld[j];
        a.epilogue = s.sage() ? SPMM_ADD_MASK : SPMM_MASK;
        a.mask_scale = st->mask_scale();
        a.aux = st->cur[j];
        a.aux_ld = s.dims[j];
        HIP_TRY(st, run_spmm(st, a, true, k, cd, cd, stream, 2, j));
      } else {
        a.out = st->grad_in;
        a.out_ld = s.dims[0];
        a.out_row0 = 0;
        a.epilogue = s.sage() ? SPMM_ADD : SPMM_PLAIN;
        HIP_TRY(st, run_spmm(st, a, true, k, cd, st->level_dtype(0), stream, 2, j));
      }
    }
    gi ^= 1;
  }
  return end_of_pass();
}
GNNSTAGE_GUARD_INT

extern "C" int update_history(gnnstage_t *st, void *hip_stream) try {
  if (!st) return GNNSTAGE_EINVAL;
  const Shape &s = st->s;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (st->cur_stale)
    return fail(st, GNNSTAGE_EORDER, "the current levels hold stale rows until a complete pass follows gnnstage_update_history_swap");
  Timed t(st, stream, 5);
  for (int j = 0; j < s.L; ++j) {
    if (st->hist[j] == st->cur[j]) continue;
    HIP_TRY(st, launch_copy(st->cur[j], st->hist[j], (size_t)s.n * s.dims[j] * st->level_elt(j), stream));
  }
  return GNNSTAGE_OK;
}
GNNSTAGE_GUARD_INT

extern "C" int gnnstage_update_history_swap(gnnstage_t *st, void *hip_stream) try {
  if (!st) return GNNSTAGE_EINVAL;
  const Shape &s = st->s;
  if ((int)st->order.size() != s.K || (st->n_bwd > 0 && st->n_bwd < s.K) || st->cur_stale)
    return fail(st, GNNSTAGE_EORDER, "the levels trade places only behind a complete pass");
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  Timed t(st, stream, 5);
  if (st->hist[0] != st->cur[0])  // level 0 is written by the caller: it keeps its buffers
    HIP_TRY(st, launch_copy(st->cur[0], st->hist[0], (size_t)s.n * s.dims[0] * st->level_elt(0), stream));
  for (int j = 1; j < s.L; ++j)
    if (st->hist[j] != st->cur[j]) {
      std::swap(st->hist[j], st->cur[j]);
      st->cur_stale = true;
    }
  return GNNSTAGE_OK;
}
GNNSTAGE_GUARD_INT

extern "C" int gnnstage_level_buffers(const gnnstage_t *st, int32_t level, void **cur, void **hist) {
  if (!st || level < 0 || level > st->s.L) return GNNSTAGE_EINVAL;
  if (cur) *cur = st->cur[(size_t)level];
  if (hist) *hist = level < st->s.L ? st->hist[(size_t)level] : nullptr;
  return GNNSTAGE_OK;
}

extern "C" int gnnstage_debug_select_counts(gnnstage_t *st, int32_t k, int32_t *out) try {
  if (!st || !out) return GNNSTAGE_EINVAL;
  const Shape &s = st->s;
  if (k < 0 || k >= s.K) return fail(st, GNNSTAGE_ERANGE, "chunk id out of range");
  ChunkMask m = st->fmask;
  mask_set(m, k);
  const uint32_t vb = (uint32_t)st->vbits;
  for (int64_t v = s.chunk_ptr[k]; v < s.chunk_ptr[k + 1]; ++v) {
    int32_t c = 0;
    for (int64_t e = st->h_row_ptr[v]; e < st->h_row_ptr[v + 1]; ++e) c += mask_test(m, st->h_pcol[(size_t)e] >> vb) ? 1 : 0;
    out[v - s.chunk_ptr[k]] = c;
  }
  return GNNSTAGE_OK;
}
GNNSTAGE_GUARD_INT

extern "C" int gnnstage_layer_order(const gnnstage_t *st, int32_t layer) {
  if (!st || layer < 0 || layer >= st->s.L) return GNNSTAGE_EINVAL;
  return st->s.tf[layer] ? 1 : 0;
}

extern "C" int gnnstage_set_dropout_rate(gnnstage_t *st, float dropout_p) {
  if (!st) return GNNSTAGE_EINVAL;
  if ((!st->order.empty() && (int)st->order.size() < st->s.K) || (st->n_bwd > 0 && st->n_bwd < st->s.K))
    return fail(st, GNNSTAGE_EORDER, "the dropout rate cannot change inside a forward or a backward pass");
  if (!(dropout_p >= 0.f && dropout_p < 1.f)) return fail(st, GNNSTAGE_EINVAL, "dropout_p must be in [0, 1)");
  if (dropout_p > 0.f && st->s.variant == GNNSTAGE_GCNII) return fail(st, GNNSTAGE_EINVAL, "no dropout in GCNII layers");
  st->next_dropout_p = dropout_p;  // latched by the next pass's first forward call
  return GNNSTAGE_OK;
}

extern "C" int gnnstage_set_dropout_seed(gnnstage_t *st, uint64_t seed) {
  if (!st) return GNNSTAGE_EINVAL;
  if ((!st->order.empty() && (int)st->order.size() < st->s.K) || (st->n_bwd > 0 && st->n_bwd < st->s.K))
    return fail(st, GNNSTAGE_EORDER, "the dropout seed cannot change inside a forward or a backward pass");
  st->next_dropout_seed = seed;  // latched by the next pass's first forward call
  return GNNSTAGE_OK;
}

extern "C" int64_t gnnstage_query(const gnnstage_t *st, int32_t what, int32_t index) {
  if (!st) return GNNSTAGE_EINVAL;
  const Shape &s = st->s;
  switch (what) {
    case GNNSTAGE_Q_VERTICES: return s.n;
    case GNNSTAGE_Q_CHUNKS: return s.K;
    case GNNSTAGE_Q_LAYERS: return s.L;
    case GNNSTAGE_Q_DTYPE: return s.dtype;
    case GNNSTAGE_Q_LEVEL0_F32: return s.level0_f32;
    case GNNSTAGE_Q_VARIANT: return s.variant;
    case GNNSTAGE_Q_NEED_INPUT_GRAD: return s.need_input_grad;
    case GNNSTAGE_Q_WIDTH: return (index >= 0 && index <= s.L) ? s.dims[(size_t)index] : GNNSTAGE_EINVAL;
    case GNNSTAGE_Q_CHUNK_PTR: return (index >= 0 && index <= s.K) ? s.chunk_ptr[(size_t)index] : GNNSTAGE_EINVAL;
    default: return GNNSTAGE_EINVAL;
  }
}

extern "C" void *gnnstage_buffer(const gnnstage_t *st, int32_t which, int32_t index) {
  if (!st) return nullptr;
  switch (which) {
    case GNNSTAGE_B_CUR: return (index >= 0 && index <= st->s.L) ? st->cur[(size_t)index] : nullptr;
    case GNNSTAGE_B_HIST: return (index >= 0 && index < st->s.L) ? st->hist[(size_t)index] : nullptr;
    case GNNSTAGE_B_GRAD_IN: return st->s.need_input_grad ? st->grad_in : nullptr;
    default: return nullptr;
  }
}

extern "C" int gnnstage_profile_enable(gnnstage_t *st, int32_t on) {
  if (!st) return GNNSTAGE_EINVAL;
  st->prof.kinds = on != 0 ? (1u << GNNSTAGE_NKINDS) - 1u : 0u;
  return GNNSTAGE_OK;
}

extern "C" int gnnstage_profile_select(gnnstage_t *st, uint32_t kind_mask) {
  if (!st || (kind_mask >> GNNSTAGE_NKINDS) != 0) return GNNSTAGE_EINVAL;
  st->prof.kinds = kind_mask;
  return GNNSTAGE_OK;
}

extern "C" int gnnstage_profile_read(gnnstage_t *st, int32_t kind, int32_t layer, double *ms, int64_t *launches) try {
  if (!st || kind < 0 || kind >= GNNSTAGE_NKINDS || layer >= st->s.L) return GNNSTAGE_EINVAL;
  if (hipDeviceSynchronize() != hipSuccess) return fail(st, GNNSTAGE_EHIP, "device synchronisation failed");
  st->prof.collect();
  double t = 0;
  int64_t n = 0;
  const int L1 = st->s.L + 1;
  for (int j = 0; j < L1; ++j) {
    if (layer >= 0 && j != layer) continue;
    t += st->prof.ms[(size_t)kind * L1 + j];
    n += st->prof.launches[(size_t)kind * L1 + j];
  }
  if (ms) *ms = t;
  if (launches) *launches = n;
  return GNNSTAGE_OK;
}
GNNSTAGE_GUARD_INT

extern "C" int gnnstage_profile_reset(gnnstage_t *st) try {
  if (!st) return GNNSTAGE_EINVAL;
  if (hipDeviceSynchronize() != hipSuccess) return fail(st, GNNSTAGE_EHIP, "device synchronisation failed");
  st->prof.collect();
  st->prof.init(st->s.L);
  return GNNSTAGE_OK;
}
GNNSTAGE_GUARD_INT
