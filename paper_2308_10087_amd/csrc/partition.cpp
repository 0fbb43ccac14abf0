// Chunk partitioner: Algorithm 1's first step ("partition V into K chunks"), locality-aware as Section 3.3 asks.
// Host only.  The heuristic is restreaming FENNEL: Tsourakakis et al. (WSDM 2014) place the vertices one by one
// into the part that maximises  |N(v) in P_i| - alpha * gamma * |P_i|^(gamma - 1)  among the parts with room,
// gamma = 3/2, alpha = balance * sqrt(K) * m / n^(3/2); Nishimura and Ugander (KDD 2013) stream the vertices again,
// each one leaving its part before it is scored against the parts as they stand.  Ties go to the lowest part,
// vertices arrive in index order, self-loops are ignored.  The parts become the chunks: vertices are renumbered
// part by part, keeping the index order inside a part.
// Balance is counted in vertices or (by_entries) in entries of the index, which is what a chunk costs to aggregate:
// vertex v then weighs its row length, n becomes the total weight W in alpha and in the capacity, and the balance
// term of v is multiplied by its weight.  A part is open while it is below the capacity.
#include <stdint.h>
#include "guard.h"

#include <cmath>
#include <vector>

#include "../../include/gnnstage.h"

extern "C" int gnnstage_partition_chunks(int64_t n, const int64_t *row_ptr, const int32_t *col_idx, int32_t n_chunks,
                                         int32_t passes, double slack, double balance, int32_t by_entries, int32_t *part,
                                         int32_t *perm, int64_t *chunk_ptr) try {
  if (n <= 0 || !row_ptr || n_chunks <= 0 || passes <= 0 || !part || !perm || !chunk_ptr) return GNNSTAGE_EINVAL;
  if (!(slack >= 1.0) || !(balance >= 0.0) || n > INT32_MAX) return GNNSTAGE_EINVAL;
  const int64_t nnz = row_ptr[n];
  if (nnz > 0 && !col_idx) return GNNSTAGE_EINVAL;
  const int K = n_chunks;
  int64_t off_diagonal = 0;
  for (int64_t v = 0; v < n; ++v) {
    if (row_ptr[v] > row_ptr[v + 1]) return GNNSTAGE_EINVAL;
    for (int64_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
      if (col_idx[e] < 0 || col_idx[e] >= n) return GNNSTAGE_EINVAL;
      off_diagonal += col_idx[e] != v;
    }
  }
  const double m = (double)off_diagonal / 2.0;  // a symmetric index lists every edge twice
  const int64_t total_w = by_entries ? nnz : n;
  if (total_w <= 0) return GNNSTAGE_EINVAL;
  const double alpha = balance * (std::sqrt((double)K) * m / ((double)total_w * std::sqrt((double)total_w)));
  const int64_t cap = (int64_t)std::ceil(slack * (double)total_w / (double)K);
  std::vector<int64_t> size((size_t)K, 0), count((size_t)K, 0);
  std::vector<int32_t> cnt((size_t)K, 0), touched;
  for (int64_t v = 0; v < n; ++v) part[v] = -1;
  for (int p = 0; p < passes; ++p) {
    for (int64_t v = 0; v < n; ++v) {
      const int64_t w = by_entries ? row_ptr[v + 1] - row_ptr[v] : 1;
      if (part[v] >= 0) {  // restreaming: v leaves its part before it is scored
        size[(size_t)part[v]] -= w;
        count[(size_t)part[v]] -= 1;
        part[v] = -1;
      }
      touched.clear();
      for (int64_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
        const int64_t u = col_idx[e];
        if (u == v || part[u] < 0) continue;
        if (cnt[(size_t)part[u]]++ == 0) touched.push_back(part[u]);
      }
      int best = -1;
      double best_score = 0.0;
      for (int i = 0; i < K; ++i) {
        if (size[(size_t)i] >= cap) continue;
        const double score = (double)cnt[(size_t)i] - alpha * 1.5 * std::sqrt((double)size[(size_t)i]) * (double)w;
        if (best < 0 || score > best_score) {
          best = i;
          best_score = score;
        }
      }
      for (int32_t i : touched) cnt[(size_t)i] = 0;
      part[v] = best;  // the capacities add up to at least the total weight, so some part is always open
      size[(size_t)best] += w;
      count[(size_t)best] += 1;
    }
  }
  chunk_ptr[0] = 0;
  for (int i = 0; i < K; ++i) chunk_ptr[i + 1] = chunk_ptr[i] + count[(size_t)i];
  std::vector<int64_t> next(chunk_ptr, chunk_ptr + K);
  for (int64_t v = 0; v < n; ++v) perm[v] = (int32_t)next[(size_t)part[v]]++;
  return GNNSTAGE_OK;
}
GNNSTAGE_GUARD_INT

// The same graph with vertex `old` renamed perm[old]; columns ascending inside every row.  Row v of the output
// is row inverse(v) of the input.  out_ptr: n + 1, out_idx: nnz.
extern "C" int gnnstage_permute_csr(int64_t n, const int64_t *row_ptr, const int32_t *col_idx, const int32_t *perm,
                                    int64_t *out_ptr, int32_t *out_idx) try {
  if (n <= 0 || !row_ptr || !perm || !out_ptr || (row_ptr[n] > 0 && (!col_idx || !out_idx))) return GNNSTAGE_EINVAL;
  std::vector<int32_t> inverse((size_t)n, -1);
  for (int64_t v = 0; v < n; ++v) {
    if (perm[v] < 0 || perm[v] >= n || inverse[(size_t)perm[v]] >= 0) return GNNSTAGE_EINVAL;  // not a permutation
    inverse[(size_t)perm[v]] = (int32_t)v;
  }
  out_ptr[0] = 0;
  for (int64_t w = 0; w < n; ++w) {
    const int64_t v = inverse[(size_t)w];
    out_ptr[w + 1] = out_ptr[w] + (row_ptr[v + 1] - row_ptr[v]);
  }
  // counting sort by new column: visit the new columns in ascending order and append to the new rows that list them
  int64_t t_nnz = row_ptr[n];
  std::vector<int64_t> t_ptr((size_t)n + 1, 0);
  std::vector<int32_t> t_row((size_t)t_nnz);
  if (gnnstage_plan_transpose(n, row_ptr, col_idx, t_ptr.data(), t_row.data(), nullptr) != GNNSTAGE_OK) return GNNSTAGE_EINVAL;
  std::vector<int64_t> fill(out_ptr, out_ptr + n);
  for (int64_t wc = 0; wc < n; ++wc) {      // new column id
    const int64_t u = inverse[(size_t)wc];  // old column id
    for (int64_t p = t_ptr[(size_t)u]; p < t_ptr[(size_t)u + 1]; ++p) {
      const int64_t w = perm[t_row[(size_t)p]];  // new id of the row that lists u
      out_idx[fill[(size_t)w]++] = (int32_t)wc;
    }
  }
  return GNNSTAGE_OK;
}
GNNSTAGE_GUARD_INT
