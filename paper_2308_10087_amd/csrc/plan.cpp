// Host-only integer bookkeeping of the stage: transposed index, packed index words and the
// launch schedule of an aggregation.  No GPU calls here, so all of it can be checked on a CPU.
#include <stdint.h>
#include "guard.h"

#include <vector>

#include <algorithm>
#include <numeric>
#include <thread>
#include <utility>

#include "../../include/gnnstage.h"
#include "plan.h"

extern "C" int gnnstage_plan_transpose(int64_t n, const int64_t *row_ptr, const int32_t *col_idx, int64_t *t_ptr,
                                       int32_t *t_row, int64_t *t_edge) try {
  if (n < 0 || !row_ptr || !t_ptr || (row_ptr[n] > 0 && (!col_idx || !t_row))) return GNNSTAGE_EINVAL;
  const int64_t nnz = row_ptr[n];
  for (int64_t i = 0; i <= n; ++i) t_ptr[i] = 0;
  for (int64_t e = 0; e < nnz; ++e) {
    const int64_t u = col_idx[e];
    if (u < 0 || u >= n) return GNNSTAGE_EINVAL;
    t_ptr[u + 1]++;
  }
  for (int64_t i = 0; i < n; ++i) t_ptr[i + 1] += t_ptr[i];
  std::vector<int64_t> next(t_ptr, t_ptr + n);
  // rows are visited in ascending order, so every column's row list comes out ascending
  for (int64_t v = 0; v < n; ++v) {
    for (int64_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
      const int64_t p = next[col_idx[e]]++;
      t_row[p] = (int32_t)v;
      if (t_edge) t_edge[p] = e;
    }
  }
  return GNNSTAGE_OK;
}
GNNSTAGE_GUARD_INT

static int bits_for(int64_t count) {  // bits needed to represent ids 0 .. count-1
  int b = 0;
  while (((int64_t)1 << b) < count) ++b;
  return b;
}

extern "C" int gnnstage_plan_pack(int64_t n, int64_t nnz, const int32_t *idx, int32_t n_chunks,
                                  const int64_t *chunk_ptr, uint32_t *packed, int32_t *vbits_out) try {
  if (n <= 0 || nnz < 0 || n_chunks <= 0 || !chunk_ptr || !vbits_out) return GNNSTAGE_EINVAL;
  int vbits = bits_for(n);
  if (vbits < 1) vbits = 1;
  const int cbits = bits_for(n_chunks);
  if (vbits > 31 || vbits + cbits > 32) return GNNSTAGE_ENOTSUP;
  *vbits_out = vbits;
  if (!packed) return GNNSTAGE_OK;
  if (nnz > 0 && !idx) return GNNSTAGE_EINVAL;
  std::vector<int32_t> chunk_of((size_t)n);
  for (int32_t c = 0; c < n_chunks; ++c) {
    if (chunk_ptr[c] > chunk_ptr[c + 1] || chunk_ptr[c] < 0 || chunk_ptr[c + 1] > n) return GNNSTAGE_EINVAL;
    for (int64_t v = chunk_ptr[c]; v < chunk_ptr[c + 1]; ++v) chunk_of[(size_t)v] = c;
  }
  if (chunk_ptr[0] != 0 || chunk_ptr[n_chunks] != n) return GNNSTAGE_EINVAL;
  for (int64_t e = 0; e < nnz; ++e) {
    const int64_t u = idx[e];
    if (u < 0 || u >= n) return GNNSTAGE_EINVAL;
    packed[e] = (uint32_t)u | ((uint32_t)chunk_of[(size_t)u] << vbits);
  }
  return GNNSTAGE_OK;
}
GNNSTAGE_GUARD_INT

namespace {
struct Task {
  int32_t row;
  int64_t e0;
  int32_t ne;
  int32_t slot;
};
}  // namespace

extern "C" int64_t gnnstage_plan_tasks(const int64_t *ptr, const int32_t *idx, int64_t n_vertices, int64_t row_begin,
                                       int64_t row_end, int32_t split_edges, int32_t n_classes,
                                       const int64_t *class_lo, int32_t class_min_row, const uint8_t *force_slot,
                                       int64_t capacity, int32_t *task_row, int64_t *task_e0, int32_t *task_ne,
                                       int32_t *task_slot, int64_t *n_slots_out, int64_t *class_off,
                                       uint8_t *slot_class) try {
  if (!ptr || row_begin > row_end || split_edges <= 0 || n_classes < 1 || n_classes > 64 || n_vertices <= 0)
    return GNNSTAGE_EINVAL;
  const bool classes = n_classes > 1 && idx != nullptr;
  // class q = source ids [lo[q], lo[q + 1]); without explicit bounds: equal id ranges
  std::vector<int64_t> lo((size_t)n_classes + 1);
  for (int q = 0; q <= n_classes; ++q)
    lo[(size_t)q] = class_lo ? class_lo[q] : ((int64_t)q * n_vertices + n_classes - 1) / n_classes;
  // With explicit bounds the classes may end before n_vertices: ids from lo[n_classes] on belong to no class
  const int64_t cls_end = lo[(size_t)n_classes];
  if (lo[0] != 0 || cls_end > n_vertices || (!class_lo && cls_end != n_vertices)) return GNNSTAGE_EINVAL;
  for (int q = 0; q < n_classes; ++q)
    if (lo[(size_t)q] > lo[(size_t)q + 1]) return GNNSTAGE_EINVAL;
  auto cls_of = [&](int64_t u) {  // last q with lo[q] <= u
    int a = 0, b = n_classes;
    while (b - a > 1) {
      const int m = (a + b) / 2;
      if (lo[(size_t)m] <= u) a = m; else b = m;
    }
    return (int64_t)a;
  };
  std::vector<std::vector<Task>> by_class(classes ? n_classes : 1);
  std::vector<Task> pieces, whole;  // pieces without a class, whole rows
  int64_t slots = 0;
  auto cut = [&](std::vector<Task> &q, int64_t r, int64_t b, int64_t e) {
    for (int64_t off = b; off < e; off += split_edges) {
      const int64_t m = e - off < split_edges ? e - off : split_edges;
      q.push_back(Task{(int32_t)r, off, (int32_t)m, (int32_t)slots});
      ++slots;
    }
  };
  for (int64_t r = row_begin; r < row_end; ++r) {
    const int64_t b = ptr[r], e = ptr[r + 1], len = e - b;
    const bool by_src = classes && len >= class_min_row;
    const bool forced = force_slot && force_slot[r];  // the row's sum has further parts: no task may finish it
    if (forced && len == 0) continue;
    if (!by_src && len <= split_edges && !forced) {  // empty rows included: they still write zeros
      whole.push_back(Task{(int32_t)r, b, (int32_t)len, -1});
      continue;
    }
    if (!by_src) {
      cut(pieces, r, b, e);
      continue;
    }
    // maximal runs of entries whose source falls in the same id range (contiguous when the row is sorted);
    // a row whose columns are so unsorted that it has more runs than classes is cut without classes.
    // Ids beyond the last class form one more run (class index n_classes) whose pieces carry no class.
    auto cls_or_none = [&](int64_t u) { return u >= cls_end ? (int64_t)n_classes : cls_of(u); };
    auto in_run = [&](int64_t u, int64_t q) {
      return q == n_classes ? u >= cls_end : (u >= lo[(size_t)q] && u < lo[(size_t)q + 1]);
    };
    int64_t runs = 1, prev = cls_or_none(idx[b]);
    for (int64_t x = b + 1; x < e && runs <= n_classes + 1; ++x) {
      const int64_t q = in_run(idx[x], prev) ? prev : cls_or_none(idx[x]);
      if (q != prev) ++runs;
      prev = q;
    }
    if (runs > n_classes + 1) {
      cut(pieces, r, b, e);
      continue;
    }
    int64_t s0 = b;
    while (s0 < e) {
      const int64_t cls = cls_or_none(idx[s0]);
      int64_t s1 = s0 + 1;
      while (s1 < e && in_run(idx[s1], cls)) ++s1;
      cut(cls == n_classes ? pieces : by_class[(size_t)cls], r, s0, s1);
      s0 = s1;
    }
  }
  // Emission, class-major: [class 0 pieces] ... [class C-1 pieces] [other pieces] [whole rows].  Which
  // workgroups serve which class is decided at launch time (one class per XCD when all are active).
  std::vector<Task> out;
  out.reserve(pieces.size() + whole.size() + (size_t)slots);
  if (classes) {
    // Inside a class the longest pieces go first: the waves of an XCD then work on pieces of similar length at any
    // time, and since every piece walks its class's source range upwards they sweep that range together (what one
    // wave brings into the L2 the others find there); it is also the better packing order for the tail.  Pieces
    // without a class and whole rows stay in row order: their output rows and metadata are then neighbours.
    auto longer = [](const Task &x, const Task &y) { return x.ne > y.ne; };
    for (auto &v : by_class) std::stable_sort(v.begin(), v.end(), longer);
  }
  for (size_t c = 0; c < by_class.size(); ++c) {
    if (class_off) class_off[c] = (int64_t)out.size();
    out.insert(out.end(), by_class[c].begin(), by_class[c].end());
    if (slot_class)
      for (const Task &t : by_class[c]) slot_class[t.slot] = (uint8_t)(classes ? c : 255);
  }
  if (class_off) {
    for (int c = (int)by_class.size(); c <= n_classes; ++c) class_off[c] = (int64_t)out.size();
    if (!classes) class_off[0] = 0, class_off[n_classes] = 0;  // no class section at all
  }
  if (slot_class)
    for (const Task &t : pieces) slot_class[t.slot] = 255;
  out.insert(out.end(), pieces.begin(), pieces.end());
  out.insert(out.end(), whole.begin(), whole.end());

  const int64_t t = (int64_t)out.size();
  if (n_slots_out) *n_slots_out = slots;
  if (task_row && task_e0 && task_ne && task_slot) {
    if (t > capacity) return GNNSTAGE_ENOMEM;
    for (int64_t i = 0; i < t; ++i) {
      task_row[i] = out[(size_t)i].row;
      task_e0[i] = out[(size_t)i].e0;
      task_ne[i] = out[(size_t)i].ne;
      task_slot[i] = out[(size_t)i].slot;
    }
  }
  return t;
}
GNNSTAGE_GUARD_INT64

// ---- dense blocks ------------------------------------------------------------------------------
bool build_dense_plan(const int64_t *ptr, const int32_t *idx, int64_t n, int K, const int64_t *chunk_ptr,
                      int min_nnz, double min_share, DensePlan &out, int item_blocks, int64_t max_items, int min_nnz_many) {
  constexpr int RB = DensePlan::RB, CB = DensePlan::CB;
  out = DensePlan();
  out.n = n;
  out.K = K;
  out.nnz = ptr[n];
  const int64_t nnz = out.nnz;
  if (nnz == 0 || min_nnz <= 0) return true;
  // how often every vertex occurs as a column
  std::vector<int64_t> col_count((size_t)n, 0);
  for (int64_t e = 0; e < nnz; ++e) {
    const int64_t u = idx[e];
    if (u < 0 || u >= n) return false;
    col_count[(size_t)u]++;
  }
  // column slots: chunk by chunk, most frequent column first
  std::vector<int64_t> cb_off((size_t)K + 1, 0);
  for (int c = 0; c < K; ++c) cb_off[(size_t)c + 1] = cb_off[(size_t)c] + (chunk_ptr[c + 1] - chunk_ptr[c] + CB - 1) / CB;
  const int64_t n_cb = cb_off[(size_t)K];
  std::vector<int32_t> colslot_vertex((size_t)(n_cb * CB), -1);
  std::vector<int64_t> slot_of((size_t)n);
  std::vector<int32_t> order;
  for (int c = 0; c < K; ++c) {
    const int64_t a = chunk_ptr[c], b = chunk_ptr[c + 1];
    order.resize((size_t)(b - a));
    std::iota(order.begin(), order.end(), (int32_t)a);
    std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) { return col_count[(size_t)x] > col_count[(size_t)y]; });
    for (int64_t i = 0; i < b - a; ++i) {
      const int64_t slot = cb_off[(size_t)c] * CB + i;
      colslot_vertex[(size_t)slot] = order[(size_t)i];
      slot_of[(size_t)order[(size_t)i]] = slot;
    }
  }
  // rows of every chunk, longest first
  std::vector<int32_t> row_perm((size_t)n);
  std::vector<int64_t> rpos((size_t)n);  // position of a row inside its chunk
  for (int c = 0; c < K; ++c) {
    const int64_t a = chunk_ptr[c], b = chunk_ptr[c + 1];
    std::iota(row_perm.begin() + a, row_perm.begin() + b, (int32_t)a);
    std::stable_sort(row_perm.begin() + a, row_perm.begin() + b,
                     [&](int32_t x, int32_t y) { return ptr[x + 1] - ptr[x] > ptr[y + 1] - ptr[y]; });
    for (int64_t i = a; i < b; ++i) rpos[(size_t)row_perm[(size_t)i]] = i - a;
  }
  // pass 1: entries per block, chunk by chunk; blocks that reach min_nnz are dense
  std::vector<int64_t> chunk_blk_off((size_t)K + 1, 0);
  std::vector<int32_t> blk_rb, blk_cb;
  std::vector<int64_t> blk_cnt;
  std::vector<int32_t> counter;
  int64_t dense_entries = 0;
  for (int c = 0; c < K; ++c) {
    const int64_t a = chunk_ptr[c], b = chunk_ptr[c + 1];
    const int64_t n_rb = (b - a + RB - 1) / RB;
    chunk_blk_off[(size_t)c + 1] = chunk_blk_off[(size_t)c];
    if (n_rb == 0) continue;
    if (n_rb * n_cb > ((int64_t)1 << 26)) return true;  // block grid too large to count: no dense path (plan stays inactive)
    counter.assign((size_t)(n_rb * n_cb), 0);
    for (int64_t r = a; r < b; ++r) {
      const int64_t base = (rpos[(size_t)r] / RB) * n_cb;
      for (int64_t e = ptr[r]; e < ptr[r + 1]; ++e) counter[(size_t)(base + slot_of[(size_t)idx[e]] / CB)]++;
    }
    for (int64_t k = 0; k < n_rb * n_cb; ++k)
      if (counter[(size_t)k] >= min_nnz) {
        blk_rb.push_back((int32_t)(k / n_cb));
        blk_cb.push_back((int32_t)(k % n_cb));
        blk_cnt.push_back(counter[(size_t)k]);
        dense_entries += counter[(size_t)k];
      }
    chunk_blk_off[(size_t)c + 1] = (int64_t)blk_rb.size();
  }
  // Threshold per row chunk: the low one while the chunk's items fit one round of workgroups (blocks are sorted by
  // chunk, then row block, so the items of a chunk are runs of equal row block cut every item_blocks blocks).
  out.min_nnz_used.assign((size_t)K, min_nnz);
  if (max_items > 0 && item_blocks > 0 && min_nnz_many > min_nnz) {
    std::vector<int64_t> off((size_t)K + 1, 0);
    size_t w = 0;
    dense_entries = 0;
    for (int c = 0; c < K; ++c) {
      auto items_at = [&](int t) {
        int64_t items = 0, run = 0;
        int32_t rb = -1;
        for (int64_t i = chunk_blk_off[(size_t)c]; i < chunk_blk_off[(size_t)c + 1]; ++i) {
          if (blk_cnt[(size_t)i] < t) continue;
          if (blk_rb[(size_t)i] != rb || run == item_blocks) {
            ++items;
            run = 0;
            rb = blk_rb[(size_t)i];
          }
          ++run;
        }
        return items;
      };
      // the lowest rung of a 5 % ladder from min_nnz at which the chunk fits one round; min_nnz_many if none below it does
      int threshold = min_nnz;
      while (threshold < min_nnz_many && items_at(threshold) > max_items) threshold = std::max(threshold + 1, (int)(threshold * 1.05));
      if (threshold > min_nnz_many) threshold = min_nnz_many;
      out.min_nnz_used[(size_t)c] = threshold;
      for (int64_t i = chunk_blk_off[(size_t)c]; i < chunk_blk_off[(size_t)c + 1]; ++i)
        if (blk_cnt[(size_t)i] >= threshold) {
          blk_rb[w] = blk_rb[(size_t)i];
          blk_cb[w] = blk_cb[(size_t)i];
          blk_cnt[w] = blk_cnt[(size_t)i];
          dense_entries += blk_cnt[w];
          ++w;
        }
      off[(size_t)c + 1] = (int64_t)w;
    }
    blk_rb.resize(w);
    blk_cb.resize(w);
    blk_cnt.resize(w);
    chunk_blk_off.swap(off);
  }
  if (blk_rb.empty() || (double)dense_entries < min_share * (double)nnz) return true;
  // pass 2: split the entries
  const int64_t nb = (int64_t)blk_rb.size();
  out.active = true;
  out.blk_e0.assign((size_t)nb + 1, 0);
  for (int64_t i = 0; i < nb; ++i) out.blk_e0[(size_t)i + 1] = out.blk_e0[(size_t)i] + blk_cnt[(size_t)i];
  out.ent_pos.resize((size_t)dense_entries);
  out.ent_orig.resize((size_t)dense_entries);
  out.rem_ptr.assign((size_t)n + 1, 0);
  out.rem_idx.reserve((size_t)(nnz - dense_entries));
  out.rem_orig.reserve((size_t)(nnz - dense_entries));
  std::vector<int64_t> cursor(out.blk_e0.begin(), out.blk_e0.end() - 1);
  std::vector<int64_t> block_of;  // block index + 1 per (row block, column block) of the current chunk
  for (int c = 0; c < K; ++c) {
    const int64_t a = chunk_ptr[c], b = chunk_ptr[c + 1];
    const int64_t n_rb = (b - a + RB - 1) / RB;
    block_of.assign((size_t)(n_rb * n_cb), 0);
    for (int64_t i = chunk_blk_off[(size_t)c]; i < chunk_blk_off[(size_t)c + 1]; ++i)
      block_of[(size_t)((int64_t)blk_rb[(size_t)i] * n_cb + blk_cb[(size_t)i])] = i + 1;
    for (int64_t r = a; r < b; ++r) {
      const int64_t rb = rpos[(size_t)r] / RB, rl = rpos[(size_t)r] % RB;
      for (int64_t e = ptr[r]; e < ptr[r + 1]; ++e) {
        const int64_t slot = slot_of[(size_t)idx[e]];
        const int64_t bi = block_of[(size_t)(rb * n_cb + slot / CB)];
        if (bi > 0) {
          const int64_t at = cursor[(size_t)(bi - 1)]++;
          out.ent_pos[(size_t)at] = (uint16_t)((rl << 8) | (slot % CB));
          out.ent_orig[(size_t)at] = e;
        } else {
          out.rem_idx.push_back(idx[e]);
          out.rem_orig.push_back(e);
        }
      }
      out.rem_ptr[(size_t)r + 1] = (int64_t)out.rem_idx.size();
    }
  }
  out.row_perm.swap(row_perm);
  out.cb_off.swap(cb_off);
  out.colslot_vertex.swap(colslot_vertex);
  out.chunk_blk_off.swap(chunk_blk_off);
  out.blk_rb.swap(blk_rb);
  out.blk_cb.swap(blk_cb);
  return true;
}

struct gnnstage_dense_plan {
  DensePlan p;
};

static int create_dense_plan(const int64_t *ptr, const int32_t *idx, int64_t n_vertices, int32_t n_chunks, const int64_t *chunk_ptr,
                             int32_t min_nnz, double min_share, int32_t item_blocks, int64_t max_items, int32_t min_nnz_many,
                             gnnstage_dense_plan **out) {
  if (!ptr || !chunk_ptr || !out || n_vertices <= 0 || n_chunks <= 0 || (ptr[n_vertices] > 0 && !idx)) return GNNSTAGE_EINVAL;
  if (chunk_ptr[0] != 0 || chunk_ptr[n_chunks] != n_vertices) return GNNSTAGE_EINVAL;
  for (int c = 0; c < n_chunks; ++c)
    if (chunk_ptr[c] > chunk_ptr[c + 1]) return GNNSTAGE_EINVAL;
  gnnstage_dense_plan *h = new gnnstage_dense_plan();
  if (!build_dense_plan(ptr, idx, n_vertices, n_chunks, chunk_ptr, min_nnz, min_share, h->p, item_blocks, max_items, min_nnz_many)) {
    delete h;
    return GNNSTAGE_EINVAL;
  }
  *out = h;
  return GNNSTAGE_OK;
}

extern "C" int gnnstage_dense_plan_create(const int64_t *ptr, const int32_t *idx, int64_t n_vertices, int32_t n_chunks,
                                          const int64_t *chunk_ptr, int32_t min_nnz, double min_share,
                                          gnnstage_dense_plan **out) try {
  return create_dense_plan(ptr, idx, n_vertices, n_chunks, chunk_ptr, min_nnz, min_share, 0, 0, 0, out);
}
GNNSTAGE_GUARD_INT

extern "C" int gnnstage_dense_plan_create_capped(const int64_t *ptr, const int32_t *idx, int64_t n_vertices, int32_t n_chunks,
                                                 const int64_t *chunk_ptr, int32_t min_nnz, double min_share, int32_t item_blocks,
                                                 int64_t max_items, int32_t min_nnz_many, gnnstage_dense_plan **out) try {
  if (item_blocks <= 0 || max_items <= 0 || min_nnz_many < min_nnz) return GNNSTAGE_EINVAL;
  return create_dense_plan(ptr, idx, n_vertices, n_chunks, chunk_ptr, min_nnz, min_share, item_blocks, max_items, min_nnz_many, out);
}
GNNSTAGE_GUARD_INT

extern "C" int64_t gnnstage_dense_plan_get(const gnnstage_dense_plan *h, int32_t what, const void **data) try {
  if (!h || !data) return GNNSTAGE_EINVAL;
  const DensePlan &p = h->p;
#define GIVE(v)                 \
  do {                          \
    *data = (v).data();         \
    return (int64_t)(v).size(); \
  } while (0)
  switch (what) {
    case 0: GIVE(p.rem_ptr);
    case 1: GIVE(p.rem_idx);
    case 2: GIVE(p.rem_orig);
    case 3: GIVE(p.row_perm);
    case 4: GIVE(p.cb_off);
    case 5: GIVE(p.colslot_vertex);
    case 6: GIVE(p.chunk_blk_off);
    case 7: GIVE(p.blk_rb);
    case 8: GIVE(p.blk_cb);
    case 9: GIVE(p.blk_e0);
    case 10: GIVE(p.ent_pos);
    case 11: GIVE(p.ent_orig);
    case 12: GIVE(p.min_nnz_used);
    default: return GNNSTAGE_EINVAL;
  }
#undef GIVE
}
GNNSTAGE_GUARD_INT64

extern "C" int gnnstage_dense_plan_destroy(gnnstage_dense_plan *h) try {
  if (!h) return GNNSTAGE_EINVAL;
  delete h;
  return GNNSTAGE_OK;
}
GNNSTAGE_GUARD_INT

// ---- hotness order -------------------------------------------------------------------------------
bool build_hot_order(const int64_t *ptr, const int32_t *idx, int64_t n, int min_row, bool want_orig, HotOrder &out) {
  out = HotOrder();
  const int64_t nnz = ptr[n];
  std::vector<int64_t> count((size_t)n, 0);
  int64_t most = 0;
  for (int64_t e = 0; e < nnz; ++e) {
    const int64_t u = idx[e];
    if (u < 0 || u >= n) return false;
    most = std::max(most, ++count[(size_t)u]);
  }
  // rank by descending count, ties by ascending id: a bucket per count value, filled in id order
  std::vector<int64_t> start((size_t)most + 2, 0);  // start[c] = first rank of the vertices that occur c times
  for (int64_t u = 0; u < n; ++u) start[(size_t)count[(size_t)u]] += 1;
  int64_t at = 0;
  for (int64_t c = most; c >= 0; --c) {
    const int64_t k = start[(size_t)c];
    start[(size_t)c] = at;
    at += k;
  }
  std::vector<int32_t> rank_of((size_t)n);
  for (int64_t u = 0; u < n; ++u) rank_of[(size_t)u] = (int32_t)start[(size_t)count[(size_t)u]]++;
  out.idx.assign(idx, idx + nnz);
  out.rank.resize((size_t)nnz);
  if (want_orig) out.orig.resize((size_t)nnz);
  const unsigned hw = std::thread::hardware_concurrency();
  const int n_threads = (int)std::max(1u, std::min(16u, hw ? hw : 1u));
  auto work = [&](int t) {
    // contiguous row ranges of about equal entry counts
    const int64_t e_lo = nnz * t / n_threads, e_hi = nnz * (t + 1) / n_threads;
    int64_t r0 = std::lower_bound(ptr, ptr + n + 1, e_lo) - ptr, r1 = std::lower_bound(ptr, ptr + n + 1, e_hi) - ptr;
    if (t == 0) r0 = 0;
    if (t == n_threads - 1) r1 = n;
    std::vector<std::pair<int32_t, int64_t>> tmp;
    for (int64_t r = r0; r < r1; ++r) {
      const int64_t b = ptr[r], e = ptr[r + 1];
      if (e - b < min_row) {
        for (int64_t x = b; x < e; ++x) {
          out.rank[(size_t)x] = rank_of[(size_t)idx[x]];
          if (want_orig) out.orig[(size_t)x] = x;
        }
        continue;
      }
      tmp.clear();
      for (int64_t x = b; x < e; ++x) tmp.emplace_back(rank_of[(size_t)idx[x]], x);
      std::sort(tmp.begin(), tmp.end());  // ranks are distinct per vertex; equal ranks (a repeated entry) fall back on position
      for (int64_t x = b; x < e; ++x) {
        const auto &p = tmp[(size_t)(x - b)];
        out.rank[(size_t)x] = p.first;
        out.idx[(size_t)x] = idx[p.second];
        if (want_orig) out.orig[(size_t)x] = p.second;
      }
    }
  };
  // lower_bound on ptr may put a row that straddles a boundary into either neighbour, never into both or none:
  // thread t takes rows [first row starting at or after e_lo, first row starting at or after e_hi)
  std::vector<std::thread> pool;
  for (int t = 1; t < n_threads; ++t) pool.emplace_back(work, t);
  work(0);
  for (auto &th : pool) th.join();
  out.active = true;
  return true;
}
