// Host-only integer bookkeeping of the stage: transposed index, packed index words and the
// launch schedule of an aggregation.  No GPU calls here, so all of it can be checked on a CPU.
#include <stdint.h>

#include <vector>

#include "../../include/gnnstage.h"

extern "C" int gnnstage_plan_transpose(int64_t n, const int64_t *row_ptr, const int32_t *col_idx, int64_t *t_ptr,
                                       int32_t *t_row, int64_t *t_edge) {
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

static int bits_for(int64_t count) {  // bits needed to represent ids 0 .. count-1
  int b = 0;
  while (((int64_t)1 << b) < count) ++b;
  return b;
}

extern "C" int gnnstage_plan_pack(int64_t n, int64_t nnz, const int32_t *idx, int32_t n_chunks,
                                  const int64_t *chunk_ptr, uint32_t *packed, int32_t *vbits_out) {
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

extern "C" int64_t gnnstage_plan_tasks(const int64_t *ptr, int64_t row_begin, int64_t row_end, int32_t split_edges,
                                       int64_t capacity, int32_t *task_row, int64_t *task_e0, int32_t *task_ne,
                                       int32_t *task_slot, int64_t *n_slots_out) {
  if (!ptr || row_begin > row_end || split_edges <= 0) return GNNSTAGE_EINVAL;
  const bool fill = task_row && task_e0 && task_ne && task_slot;
  int64_t t = 0, slots = 0;
  // pass 1: pieces of long rows first, so that the biggest tasks start early
  for (int64_t r = row_begin; r < row_end; ++r) {
    const int64_t len = ptr[r + 1] - ptr[r];
    if (len <= split_edges) continue;
    for (int64_t off = 0; off < len; off += split_edges) {
      if (fill) {
        if (t >= capacity) return GNNSTAGE_ENOMEM;
        task_row[t] = (int32_t)r;
        task_e0[t] = ptr[r] + off;
        task_ne[t] = (int32_t)(len - off < split_edges ? len - off : split_edges);
        task_slot[t] = (int32_t)slots;
      }
      ++t;
      ++slots;
    }
  }
  // pass 2: every other row is one task (empty rows included: they still write zeros)
  for (int64_t r = row_begin; r < row_end; ++r) {
    const int64_t len = ptr[r + 1] - ptr[r];
    if (len > split_edges) continue;
    if (fill) {
      if (t >= capacity) return GNNSTAGE_ENOMEM;
      task_row[t] = (int32_t)r;
      task_e0[t] = ptr[r];
      task_ne[t] = (int32_t)len;
      task_slot[t] = -1;
    }
    ++t;
  }
  if (n_slots_out) *n_slots_out = slots;
  return t;
}
