// Host-side plans shared between plan.cpp (which builds them) and the stage (which uploads them).
#pragma once
#include <stdint.h>

#include <vector>

// Dense-block plan of one aggregation direction (a sparse index ptr/idx over n vertices, rows grouped
// into K chunks).  Inside a chunk the rows are ordered by length, the vertices of every chunk are
// ordered by how often they occur as a column, and the matrix is cut into RB x CB blocks in those
// orders.  Blocks with at least min_nnz entries are "dense": their entries leave the sparse index and
// are multiplied on the matrix cores as small dense products; everything else stays in the remainder.
struct DensePlan {
  static constexpr int RB = 128, CB = 64;
  int64_t n = 0, nnz = 0;
  int K = 0;
  bool active = false;  // false: no dense blocks, the remainder is the whole index (arrays below empty)
  // remainder (same rows, same column order inside a row)
  std::vector<int64_t> rem_ptr;    // n + 1
  std::vector<int32_t> rem_idx;    // column of every remainder entry
  std::vector<int64_t> rem_orig;   // its position in the original index
  // orders
  std::vector<int32_t> row_perm;        // n: chunk k occupies [chunk_ptr[k], chunk_ptr[k+1]), longest row first
  std::vector<int64_t> cb_off;          // K + 1: column blocks of chunk c are [cb_off[c], cb_off[c+1])
  std::vector<int32_t> colslot_vertex;  // cb_off[K] * CB: vertex in every column slot, -1 = padding
  // dense blocks, sorted by (row chunk, row block, column block)
  std::vector<int64_t> chunk_blk_off;   // K + 1: blocks whose rows are in chunk k
  std::vector<int32_t> blk_rb;          // row block inside its chunk (rows row_perm[chunk_ptr[k] + RB*rb ...])
  std::vector<int32_t> blk_cb;          // column block (global numbering, see cb_off)
  std::vector<int64_t> blk_e0;          // n_blocks + 1: entries of a block
  std::vector<uint16_t> ent_pos;        // (row inside the block) << 8 | column inside the block
  std::vector<int64_t> ent_orig;        // position in the original index
  std::vector<int32_t> min_nnz_used;    // K entries: the threshold the blocks of every row chunk were selected with
  int64_t n_blocks() const { return (int64_t)blk_rb.size(); }
};

// min_share: the plan is only activated when at least this share of all entries falls into dense blocks.
// max_items > 0: the dense kernel serves the blocks of a row block in items of at most item_blocks blocks, one
// workgroup per item and column half.  A launch (one row chunk) that fits one round of workgroups can afford a low
// threshold: its time is set by its longest item whatever the number of blocks.  Every chunk takes the lowest rung
// of a 5 % ladder from min_nnz at which it has at most max_items items; a chunk that does not get there below
// min_nnz_many needs several rounds, every block then costs time, and it takes min_nnz_many.
// Returns false on invalid input (an index entry outside [0, n)).
bool build_dense_plan(const int64_t *ptr, const int32_t *idx, int64_t n, int K, const int64_t *chunk_ptr,
                      int min_nnz, double min_share, DensePlan &out, int item_blocks = 0, int64_t max_items = 0,
                      int min_nnz_many = 0);

// Hotness order of one aggregation direction.  A source's hotness is how often it occurs in the index; rank 0 is
// the most often gathered vertex (ties: lower id first).  Rows with at least min_row entries get their entries
// re-ordered by ascending rank, so that the entries whose sources belong to one slice of the hottest vertices are
// one contiguous run of the row; shorter rows keep their order.  idx / rank / orig describe the index after the
// re-ordering: source id, its rank, and the entry's position in the index the order was built from.
struct HotOrder {
  bool active = false;
  std::vector<int32_t> idx, rank;
  std::vector<int64_t> orig;  // empty unless asked for
};
// Returns false on an index entry outside [0, n).
bool build_hot_order(const int64_t *ptr, const int32_t *idx, int64_t n, int min_row, bool want_orig, HotOrder &out);
