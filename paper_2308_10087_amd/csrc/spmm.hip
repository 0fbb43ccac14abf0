// Neighbour aggregation with the current-vs-history select fused into the gather
// (Algorithm 1, the AGGREGATE line; Section 3.3), and its transposed twin for the
// backward pass where unselected entries contribute zero (Section 3.4, technique 3).
//
// One wavefront per task.  A task is a whole sparse row, or a piece of a long row (power-law
// hubs are cut so that no wave owns more than a fixed number of entries; the pieces write
// fp32 partial sums that a second small kernel adds in a fixed order, so results do not
// depend on scheduling).  Two kernels share that schedule:
//  * spmm_kernel, the vector-ALU form for fp32 rows and odd widths: the 64 lanes form G = 64/LPR
//    groups of LPR lanes, each group gathers one neighbour row per step with 16/8/4-byte loads;
//    entry metadata (packed index, weight) is loaded 64 entries at a time, one per lane, and
//    broadcast through lane permutes; dropped entries are first compacted inside the wave.
//  * spmm_ring_kernel, for bf16 rows whose width is a multiple of 8: entries become address
//    records in a wave-private LDS ring and the weighted sum runs on the matrix cores.
#include "common.h"

namespace {

template <typename T, int V>
struct alignas((sizeof(T) * V) > 16 ? 16 : (sizeof(T) * V)) Pack {
  T v[V];
};

__device__ inline float to_f32(float x) { return x; }
__device__ inline float to_f32(bf16_t x) { return (float)x; }
template <typename T>
__device__ inline T from_f32(float x);
template <>
__device__ inline float from_f32<float>(float x) { return x; }
template <>
__device__ inline bf16_t from_f32<bf16_t>(float x) { return (bf16_t)x; }

// The row of the auxiliary matrix that the mixing and masking epilogues read (zeros for the others).
template <typename Tin, int VEC>
__device__ inline Pack<Tin, VEC> load_aux(const SpmmArgs &a, int64_t row, int c) {
  if (spmm_reads_aux(a.epilogue))
    return *reinterpret_cast<const Pack<Tin, VEC> *>(static_cast<const Tin *>(a.aux) + (size_t)row * a.aux_ld + c);
  Pack<Tin, VEC> z;
#pragma unroll
  for (int t = 0; t < VEC; ++t) z.v[t] = from_f32<Tin>(0.f);
  return z;
}

// Applies the epilogue to VEC consecutive columns of one output row and stores them; x is load_aux of the
// same columns (a caller with other loads in flight asks for it early).
template <typename Tin, typename Tout, int VEC>
__device__ inline void finish_cols(const SpmmArgs &a, int64_t row, int c, const float (&acc)[VEC], const Pack<Tin, VEC> &x) {
  float r[VEC];
  if (a.epilogue == SPMM_PLAIN) {
#pragma unroll
    for (int t = 0; t < VEC; ++t) r[t] = acc[t];
  } else if (a.epilogue == SPMM_BIAS_RELU) {
#pragma unroll
    for (int t = 0; t < VEC; ++t) {
      const float y = acc[t] + a.bias[c + t];
      r[t] = y > 0.f ? y : 0.f;
    }
  } else if (spmm_reads_add(a.epilogue)) {
    const Pack<Tin, VEC> y = *reinterpret_cast<const Pack<Tin, VEC> *>(
        static_cast<const Tin *>(a.add) + (size_t)(row - a.add_row0) * a.add_ld + c);
#pragma unroll
    for (int t = 0; t < VEC; ++t) {
      const float sum = acc[t] + to_f32(y.v[t]);
      r[t] = a.epilogue == SPMM_ADD ? sum : to_f32(x.v[t]) > 0.f ? sum * a.mask_scale : 0.f;
    }
  } else if (a.epilogue == SPMM_MIX) {
#pragma unroll
    // one rounding for the dominant (1 - alpha) term: with rows on the bf16 grid the exact mix often sits
    // exactly half-way between two bf16 values, and rounding the large product separately would push all
    // of those ties the same way
    for (int t = 0; t < VEC; ++t) r[t] = __builtin_fmaf(a.s_acc, acc[t], a.s_aux * to_f32(x.v[t]));
  } else {
#pragma unroll
    for (int t = 0; t < VEC; ++t) r[t] = to_f32(x.v[t]) > 0.f ? acc[t] * a.mask_scale : 0.f;
  }
  Pack<Tout, VEC> o;
#pragma unroll
  for (int t = 0; t < VEC; ++t) o.v[t] = from_f32<Tout>(r[t]);
  *reinterpret_cast<Pack<Tout, VEC> *>(static_cast<Tout *>(a.out) + (size_t)(row - a.out_row0) * a.out_ld + c) = o;
}

template <typename Tin, typename Tout, int VEC>
__device__ inline void finish_cols(const SpmmArgs &a, int64_t row, int c, const float (&acc)[VEC]) {
  finish_cols<Tin, Tout, VEC>(a, row, c, acc, load_aux<Tin, VEC>(a, row, c));
}

template <typename Tout>
__device__ inline void zero_pad_cols(const SpmmArgs &a, int64_t row, int lane) {
  const int c = a.d + lane;
  if (c < a.out_ld) static_cast<Tout *>(a.out)[(size_t)(row - a.out_row0) * a.out_ld + c] = from_f32<Tout>(0.f);
}

template <typename Tin, typename Tout, int VEC, int LPR, int NV>
__global__ __launch_bounds__(256) void spmm_kernel(const SpmmArgs a) {
  constexpr int G = 64 / LPR;
  constexpr int TILE_W = LPR * NV * VEC;
  const int lane = threadIdx.x & 63;
  const int64_t task = spmm_task_index(a, blockIdx.x, threadIdx.x >> 6);
  if (task < 0) return;  // whole wave leaves together
  const int grp = lane / LPR, lig = lane % LPR;
  const int col0 = blockIdx.y * TILE_W + lig * VEC;
  // task fields are the same for the whole wave: keep them in scalar registers, so that every loop
  // bound below is provably wave-uniform (the lane permutes need all lanes in step)
  const int64_t row = __builtin_amdgcn_readfirstlane(a.task_row[task]);
  const int64_t e0_raw = a.task_e0[task];
  const int64_t e0 = ((int64_t)__builtin_amdgcn_readfirstlane((int)(e0_raw >> 32)) << 32) |
                     (uint32_t)__builtin_amdgcn_readfirstlane((int)(e0_raw & 0xffffffff));
  const int ne = __builtin_amdgcn_readfirstlane(a.task_ne[task]);
  const int slot = __builtin_amdgcn_readfirstlane(a.task_slot[task]);
  const uint32_t vmask = (1u << a.vbits) - 1u;
  const bool drop_unsel = a.src_unsel == nullptr;
  const Tin *src_sel = static_cast<const Tin *>(a.src_sel);
  const Tin *src_unsel = static_cast<const Tin *>(a.src_unsel);
  const int d = a.d;
  const size_t ld = (size_t)a.src_ld;

  float acc[NV][VEC];
#pragma unroll
  for (int v = 0; v < NV; ++v)
#pragma unroll
    for (int t = 0; t < VEC; ++t) acc[v][t] = 0.f;

  for (int base = 0; base < ne; base += 64) {
    int n = ne - base < 64 ? ne - base : 64;
    uint32_t info = 0;
    float w = 0.f;
    bool keep = false;
    if (lane < n) {
      const int64_t e = e0 + base + lane;
      const uint32_t pc = a.pidx[e];
      const bool sel = mask_test(a.mask, pc >> a.vbits);
      keep = sel || !drop_unsel;
      info = (pc & vmask) | (sel ? 0x80000000u : 0u);
      w = a.val[e];
    }
    if (drop_unsel) {  // wave-uniform: compact the kept entries to the low lanes
      const uint64_t bal = __ballot(keep);
      const int nk = __popcll(bal);
      const int rk = __popcll(bal & ((1ull << lane) - 1ull));
      const int dest = keep ? rk : nk + (lane - rk);
      info = (uint32_t)__builtin_amdgcn_ds_permute(dest << 2, (int)info);
      w = __int_as_float(__builtin_amdgcn_ds_permute(dest << 2, __float_as_int(w)));
      n = __builtin_amdgcn_readfirstlane(nk);
    }
    for (int i = 0; i < n; i += G) {
      const int idx = i + grp;
      const int from = idx < n ? idx : i;  // past the end: re-read a valid entry with weight 0
      const uint32_t inf = (uint32_t)__shfl((int)info, from);
      float ww = __shfl(w, from);
      if (idx >= n) ww = 0.f;
      const Tin *rowp = ((inf >> 31) ? src_sel : src_unsel) + (size_t)(inf & 0x7fffffffu) * ld + col0;
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        if (col0 + v * LPR * VEC < d) {
          const Pack<Tin, VEC> x = *reinterpret_cast<const Pack<Tin, VEC> *>(rowp + v * LPR * VEC);
#pragma unroll
          for (int t = 0; t < VEC; ++t) acc[v][t] += ww * to_f32(x.v[t]);
        }
      }
    }
  }
  // add the G groups' partial rows (same columns live LPR lanes apart)
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
    for (int v = 0; v < NV; ++v)
#pragma unroll
      for (int t = 0; t < VEC; ++t) acc[v][t] += __shfl_xor(acc[v][t], off);

  if (grp == 0) {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int c = col0 + v * LPR * VEC;
      if (c < d) {
        if (slot >= 0) {
          Pack<float, VEC> o;
#pragma unroll
          for (int t = 0; t < VEC; ++t) o.v[t] = acc[v][t];
          *reinterpret_cast<Pack<float, VEC> *>(a.partial + (size_t)slot * d + c) = o;
        } else {
          finish_cols<Tin, Tout, VEC>(a, row, c, acc[v]);
        }
      }
    }
    if (slot < 0 && blockIdx.y == 0) zero_pad_cols<Tout>(a, row, lig);
  }
}

// Sums the pieces of every cut row, then applies the epilogue.  One workgroup per row: 8 phases x 32
// column vectors; phase p adds the slots p, p+8, p+16, ... (hub rows have hundreds of pieces), then the 8
// phase sums are added in order.  The order is fixed, so results are reproducible.
// A workgroup moves a few KB, so what it costs is its chain of dependent memory round trips.  There are
// two: the row's header words, then everything else at once.  Pieces that may not count (a class or an item
// that did not run in this launch holds stale sums) are loaded anyway, together with the word that says so,
// and left out by a select; the epilogue's auxiliary row is asked for before the sums.
template <typename Tin, typename Tout, int VEC>
__global__ __launch_bounds__(256) void spmm_reduce_kernel(const SpmmArgs a) {
  __shared__ float red[8][32][VEC];
  const int64_t i = blockIdx.x;
  const int ph = threadIdx.x >> 5, cv = threadIdx.x & 31;
  const bool dense = a.lr_ndense != nullptr;
  const int64_t row = a.lr_row[i];
  const int slot0 = a.lr_slot0[i], ns = a.lr_nslots[i];
  const int nd = dense ? a.lr_ndense[i] : 0;
  const int dense0 = dense ? a.lr_dense0[i] : 0, item0 = dense ? a.lr_item0[i] : 0;
  // pieces of classes that were not run in this launch (all their entries unselected) hold stale data
  const bool check = a.slot_class != nullptr && a.all_classes_active == 0;
  for (int c0 = 0; c0 < a.d; c0 += 32 * VEC) {
    const int c = c0 + cv * VEC;
    float acc[VEC];
#pragma unroll
    for (int t = 0; t < VEC; ++t) acc[t] = 0.f;
    Pack<Tin, VEC> xa;
    if (c < a.d) {
      if (ph == 0) xa = load_aux<Tin, VEC>(a, row, c);
      for (int s = ph; s < ns; s += 8) {
        const uint32_t sc = check ? a.slot_class[slot0 + s] : 32u;
        const Pack<float, VEC> x = *reinterpret_cast<const Pack<float, VEC> *>(a.partial + (size_t)(slot0 + s) * a.d + c);
        const bool use = sc >= 32u || ((a.active_classes >> sc) & 1u);
#pragma unroll
        for (int t = 0; t < VEC; ++t) acc[t] += use ? x.v[t] : 0.f;
      }
      // the row's parts from dense blocks: one partial row per item of its row block
      for (int g = ph; g < nd; g += 8) {
        bool use = true;
        if (a.drop_unselected) {  // an item without a selected chunk was not run
          const ChunkMask m = a.item_chunks[item0 + g];
          use = ((m.w[0] & a.mask.w[0]) | (m.w[1] & a.mask.w[1]) | (m.w[2] & a.mask.w[2]) | (m.w[3] & a.mask.w[3])) != 0;
        }
        const Pack<float, VEC> x =
            *reinterpret_cast<const Pack<float, VEC> *>(a.dense_partial + ((size_t)dense0 + (size_t)g * kDenseRB) * a.d + c);
#pragma unroll
        for (int t = 0; t < VEC; ++t) acc[t] += use ? x.v[t] : 0.f;
      }
    }
#pragma unroll
    for (int t = 0; t < VEC; ++t) red[ph][cv][t] = acc[t];
    __syncthreads();
    if (ph == 0 && c < a.d) {
#pragma unroll
      for (int p = 1; p < 8; ++p)
#pragma unroll
        for (int t = 0; t < VEC; ++t) acc[t] += red[p][cv][t];
      finish_cols<Tin, Tout, VEC>(a, row, c, acc, xa);
    }
    __syncthreads();
  }
  if (threadIdx.x < 64) zero_pad_cols<Tout>(a, row, threadIdx.x);
}

// ---- bf16 sources: the weighted row sum on the matrix cores ---------------------------------
// A gathered 16-byte piece (8 consecutive bf16 columns of one neighbour row) is exactly one lane's
// A-operand fragment of v_mfma_f32_16x16x32_bf16: lane l supplies A[m = l%16][k = 8*(l/16) .. +8].
// Reading m as "8-column block" and k as (neighbour slot g = l/16, column t inside the block), the
// B operand  B[8g + t][n] = w_g * [t == n % 8]  turns the instruction into
//     D[m][n] += sum_g w_g * X[u_g][8m + n % 8]
// i.e. four neighbours (one per 16-lane group) times a 128-column tile are scaled by their edge
// weights and accumulated in fp32 with no bf16->fp32 conversion and no vector FMA.  Columns n < 8 of B
// carry the upper bf16 half of the fp32 weight, columns n >= 8 the remainder, and the two halves of D
// are added at the end, so the weight keeps 16 mantissa bits.  (A non-finite input value also poisons
// the other 7 columns of its 8-column block, since 0 * inf = nan inside the dot product.)
typedef bf16_t bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) bf16x8_t global_bf16x8_t;  // a load through it is a global load

// Short rows (at most a few entries: the bulk of a power-law graph's rows, a few percent of its entries).  A wave
// per row would spend its life waiting for three dependent round trips to move a kilobyte or two, and a launch
// would need several rounds of waves.  Here every 16-lane group owns one row: a lane keeps 8 columns of each
// 128-column tile in fp32 registers and the sum runs on the vector ALU; two to four of the row's entries are in
// flight per lane.  Entries that a backward launch drops are not loaded at all.  `first` = index of the first row
// of this workgroup among the launch's short rows.
template <typename Tout, int NT, bool FULL>
__device__ __forceinline__ void spmm_short_rows(const SpmmArgs &a, int64_t first) {
  const int lane = threadIdx.x & 63, lig = lane & 15;
  const int64_t t = first + (threadIdx.x >> 4);
  if (t >= a.n_short) return;
  const int64_t task = a.n_tasks + t;  // the short rows follow the tasks of the main part
  const uint32_t vmask = (1u << a.vbits) - 1u;
  const bool drop_unsel = a.src_unsel == nullptr;
  const char *base_sel = static_cast<const char *>(a.src_sel);
  const char *base_unsel = drop_unsel ? base_sel : static_cast<const char *>(a.src_unsel);
  const size_t row_bytes = (size_t)a.src_ld * 2u;
  const int d = a.d;
  const int64_t row = a.task_row[task];
  const int64_t e0 = a.task_e0[task];
  const int ne = a.task_ne[task];
  float acc[NT][8];
#pragma unroll
  for (int h = 0; h < NT; ++h)
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[h][c] = 0.f;
  constexpr int SU = NT == 1 ? 4 : 2;  // entries in flight per lane (16 bytes x NT each)
  for (int i = 0; i < ne; i += SU) {
    bf16x8_t x[SU][NT];
    float w[SU];
#pragma unroll
    for (int u = 0; u < SU; ++u) {
      w[u] = 0.f;
#pragma unroll
      for (int h = 0; h < NT; ++h) x[u][h] = bf16x8_t{0, 0, 0, 0, 0, 0, 0, 0};
      if (i + u < ne) {
        const uint32_t pc = a.pidx[e0 + i + u];
        const bool sel = mask_test(a.mask, pc >> a.vbits);
        if (sel || !drop_unsel) {
          w[u] = a.val[e0 + i + u];
          const char *p = (sel ? base_sel : base_unsel) + (size_t)(pc & vmask) * row_bytes + (size_t)lig * 16u;
#pragma unroll
          for (int h = 0; h < NT; ++h)
            if (FULL || h * 128 + lig * 8 < d) x[u][h] = *reinterpret_cast<const bf16x8_t *>(p + h * 256);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < SU; ++u)
#pragma unroll
      for (int h = 0; h < NT; ++h)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[h][c] = __builtin_fmaf(w[u], (float)x[u][h][c], acc[h][c]);
  }
#pragma unroll
  for (int h = 0; h < NT; ++h) {
    const int c = h * 128 + lig * 8;
    if (FULL || c < d) finish_cols<bf16_t, Tout, 8>(a, row, c, acc[h]);
  }
  zero_pad_cols<Tout>(a, row, lig);
}

// Entry metadata is turned, once per entry, into a 16-byte record {row address, packed weight halves}
// and appended to a wave-private ring in LDS; unselected entries of a backward launch are simply not
// appended, so the gather loop sees one dense stream of kept entries across the 64-entry metadata
// batches.  A wave alternates between two phases.  Phase A turns KB batches of metadata (loaded during
// the previous phase B) into records.  Phase B gathers: it works in steps of four records (one per
// 16-lane group) and owns U register slots; slot u holds the pieces of step s with s % U == u.  In the
// steady loop every slot is multiplied into the accumulators and immediately refilled with the loads of
// step s + U, unconditionally, so the number of younger loads at every wait is a compile-time constant
// and U - 1 steps of gathers stay in flight while one is consumed.  Per step the vector ALU only adds
// the lane offset to the record's address and expands the weight (one byte permute, four selects).
template <typename Tout, int NT, int U, bool FULL>
__global__ __launch_bounds__(256, (NT * U <= 8) ? 7 : 1) void spmm_ring_kernel(const SpmmArgs a) {
  constexpr int TILE_W = NT * 128;
  constexpr int KB = 2;    // metadata batches per phase
  constexpr int R = 256;   // ring capacity in records: a phase appends at most 64 * KB, fewer than 8 * U are left over
  static_assert(TILE_W * sizeof(float) <= R * sizeof(u32x4_t), "the output row reuses the ring's memory");
  static_assert((U & (U - 1)) == 0 && U <= 8, "slot count");
  __shared__ u32x4_t ring_all[4][R];
  if ((int64_t)blockIdx.x >= a.n_main_blocks) {  // the workgroups behind the main part serve the short rows, 16 each
    if constexpr (NT <= 2) spmm_short_rows<Tout, NT, FULL>(a, ((int64_t)blockIdx.x - a.n_main_blocks) * 16);
    return;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t task = spmm_task_index(a, blockIdx.x, wave);
  if (task < 0) return;  // whole wave leaves together (no block-wide barrier below)
  u32x4_t *ring = ring_all[wave];
  const int g = lane >> 4, lig = lane & 15;
  const int tile0 = blockIdx.y * TILE_W;
  // Task fields are the same for the whole wave: keep them in scalar registers.  The matrix instruction
  // ignores the execution mask, so all control flow around it must be provably wave-uniform.
  const int64_t row = __builtin_amdgcn_readfirstlane(a.task_row[task]);
  const int64_t e0_raw = a.task_e0[task];
  const int64_t e0 = ((int64_t)__builtin_amdgcn_readfirstlane((int)(e0_raw >> 32)) << 32) |
                     (uint32_t)__builtin_amdgcn_readfirstlane((int)(e0_raw & 0xffffffff));
  const int ne = __builtin_amdgcn_readfirstlane(a.task_ne[task]);
  const int slot = __builtin_amdgcn_readfirstlane(a.task_slot[task]);
  const uint32_t vmask = (1u << a.vbits) - 1u;
  const bool drop_unsel = a.src_unsel == nullptr;
  const char *base_sel = static_cast<const char *>(a.src_sel) + (size_t)tile0 * 2;
  const char *base_unsel = drop_unsel ? base_sel : static_cast<const char *>(a.src_unsel) + (size_t)tile0 * 2;
  const int d = a.d;
  const uint32_t row_bytes = (uint32_t)a.src_ld * 2u;
  const uint32_t lane_off = (uint32_t)lig * 16u;
  const int pos = lig & 7;        // which element of the 8-column block this lane's B column picks
  const bool lo_part = lig >= 8;  // B columns 8..15 carry the low half of the weight
  // byte selector that moves this lane's weight half (bytes 0-1 or 2-3 of the packed word) into the
  // bf16 element `pos & 1` of a B operand word and zeroes the other element
  const uint32_t b0 = lo_part ? 2u : 0u;
  const uint32_t selw = (pos & 1) ? (((b0 + 1u) << 24) | (b0 << 16) | 0x0c0cu) : (0x0c0c0000u | ((b0 + 1u) << 8) | b0);
  const int wword = pos >> 1;
  const uint64_t mask0 = a.mask.w[0], mask1 = a.mask.w[1], mask2 = a.mask.w[2], mask3 = a.mask.w[3];

  f32x4_t acc[NT];
#pragma unroll
  for (int h = 0; h < NT; ++h) acc[h] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  const bf16x8_t zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  bf16x8_t x[U][NT];
  uint32_t wk[U];
  uint64_t rec_addr = 0;  // record of the next step to issue, read one step ahead
  uint32_t rec_w = 0;

  auto read_record = [&](int step) {
    const uint32_t *rec = reinterpret_cast<const uint32_t *>(&ring[((step << 2) + g) & (R - 1)]);
    rec_addr = *reinterpret_cast<const uint64_t *>(rec);
    rec_w = rec[2];
  };
  // gathers of step `step` into slot u; the record was read before, the following one is requested now
  // (past the last appended record this reads stale ring memory that nobody uses)
  auto issue = [&](int step, int u) {
    const global_bf16x8_t *p = reinterpret_cast<const global_bf16x8_t *>(rec_addr + lane_off);
    wk[u] = rec_w;
#pragma unroll
    for (int h = 0; h < NT; ++h) x[u][h] = (FULL || tile0 + h * 128 + lig * 8 < d) ? p[h * 16] : zero8;
    read_record(step + 1);
    // keep the slots in program order: the wait in front of a slot's product then only covers that slot's
    // own loads and leaves the younger gathers in flight
    __builtin_amdgcn_sched_barrier(0);
  };
  auto consume = [&](int u) {
    const uint32_t wbits = __builtin_amdgcn_perm(0u, wk[u], selw);
    u32x4_t bw;
    bw[0] = wword == 0 ? wbits : 0u;
    bw[1] = wword == 1 ? wbits : 0u;
    bw[2] = wword == 2 ? wbits : 0u;
    bw[3] = wword == 3 ? wbits : 0u;
    const bf16x8_t bfrag = __builtin_bit_cast(bf16x8_t, bw);
#pragma unroll
    for (int h = 0; h < NT; ++h) acc[h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x[u][h], bfrag, acc[h], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  };

  const int nb = (ne + 63) >> 6;  // metadata batches
  int bprod = 0;                  // batches turned into records so far
  int produced = 0;               // records appended so far
  int issued = 0;                 // steps whose gathers have been issued (and, between phases, multiplied)
  uint32_t pad_lo = 0, pad_hi = 0;  // address of some kept row, for the zero-weight records that fill the last step

  uint32_t pcs[KB];
  float ws[KB];
  auto prefetch = [&](int b0) {  // clamped index: lanes past the end re-read the last entry and are not kept
#pragma unroll
    for (int k = 0; k < KB; ++k) {
      int i = ((b0 + k) << 6) + lane;
      i = i < ne ? i : ne - 1;
      pcs[k] = a.pidx[e0 + i];
      ws[k] = a.val[e0 + i];
    }
  };
  if (ne > 0) prefetch(0);
  while (bprod < nb) {
    // ---- phase A: KB batches of metadata become records
#pragma unroll
    for (int k = 0; k < KB; ++k) {
      const int nraw = ne - ((bprod + k) << 6);  // entries left from this batch on (may be <= 0)
      const uint32_t pc = pcs[k];
      const float w = ws[k];
      // the chunk's bit of the processed mask, picked with register selects (no indexed access)
      const uint32_t ci = pc >> a.vbits;
      const uint64_t mlo = (ci & 64u) ? mask1 : mask0, mhi = (ci & 64u) ? mask3 : mask2;
      const bool sel = ((((ci & 128u) ? mhi : mlo) >> (ci & 63u)) & 1ull) != 0;
      const bool keep = lane < nraw && (sel || !drop_unsel);
      const uint64_t addr = reinterpret_cast<uint64_t>(sel ? base_sel : base_unsel) + (uint64_t)(pc & vmask) * row_bytes;
      const bf16_t whi = (bf16_t)w;
      const bf16_t wlo = (bf16_t)(w - (float)whi);
      const uint32_t wpk = (uint32_t)__builtin_bit_cast(uint16_t, whi) | ((uint32_t)__builtin_bit_cast(uint16_t, wlo) << 16);
      const uint64_t bal = __ballot(keep);
      const int nk = __builtin_amdgcn_readfirstlane(__popcll(bal));
      const int rk = (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
      if (keep) ring[(produced + rk) & (R - 1)] = u32x4_t{(uint32_t)addr, (uint32_t)(addr >> 32), wpk, 0u};
      if (nk > 0) {
        const int first = __builtin_amdgcn_readfirstlane(__ffsll((unsigned long long)bal) - 1);
        pad_lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)addr, first);
        pad_hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(addr >> 32), first);
      }
      produced += nk;
    }
    bprod += KB;
    const bool final = bprod >= nb;
    if (!final) prefetch(bprod);  // lands while this phase's gathers run
    if (final) {  // complete the last step with zero-weight records that point at a row of the sum
      const int padn = (-produced) & 3;
      if (lane < padn) ring[(produced + lane) & (R - 1)] = u32x4_t{pad_lo, pad_hi, 0u, 0u};
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int avail = final ? (produced + 3) >> 2 : produced >> 2;  // steps that may be issued
    const int count = avail - issued;
    if (!final && count < 2 * U) continue;  // too few kept entries for a steady loop: collect more first
    // ---- phase B: steps issued .. avail - 1
    read_record(issued);
    int k = 0;
    if (count >= 2 * U) {
#pragma unroll
      for (int u = 0; u < U; ++u) issue(issued + u, u);
      for (; k + 2 * U <= count; k += U) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          consume(u);
          issue(issued + k + U + u, u);
        }
      }
    } else {
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (u < count) issue(issued + u, u);
    }
    // steps k .. k + U - 1 (those below count) are in their slots; fewer than U further steps remain
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (k + u < count) consume(u);
      if (k + U + u < count) issue(issued + k + U + u, u);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (k + U + u < count) consume(u);
    issued = avail;
  }
  // D layout: element i of lane l is D[m = 4*(l/16) + i][n = l%16]; column = 8m + n%8, halves n<8 / n>=8
  float *rowbuf = reinterpret_cast<float *>(ring);  // every record has been read: the ring's memory is free
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int h = 0; h < NT; ++h)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float v = acc[h][i] + __shfl_xor(acc[h][i], 8);
      if (!lo_part) rowbuf[h * 128 + (4 * g + i) * 8 + pos] = v;
    }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the wave's own LDS writes have landed
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  // natural layout again: lane q owns 8 consecutive columns
#pragma unroll
  for (int r = 0; r < (NT * 16 + 63) / 64; ++r) {
    const int q = lane + 64 * r;
    const int c = tile0 + q * 8;
    if (q < NT * 16 && c < d) {
      float v[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) v[t] = rowbuf[q * 8 + t];
      if (slot >= 0) {
        Pack<float, 8> o;
#pragma unroll
        for (int t = 0; t < 8; ++t) o.v[t] = v[t];
        *reinterpret_cast<Pack<float, 8> *>(a.partial + (size_t)slot * d + c) = o;
      } else {
        finish_cols<bf16_t, Tout, 8>(a, row, c, v);
      }
    }
  }
  if (slot < 0 && blockIdx.y == 0) zero_pad_cols<Tout>(a, row, lane);
}

typedef void (*spmm_fn)(const SpmmArgs);
struct Shape {
  int vec, lpr, nv;
  spmm_fn main, reduce;
};

template <typename Tin, typename Tout, int VEC, int LPR, int NV>
constexpr Shape shape_of() {
  return Shape{VEC, LPR, NV, spmm_kernel<Tin, Tout, VEC, LPR, NV>, spmm_reduce_kernel<Tin, Tout, VEC>};
}

template <typename Tout>
const Shape *shapes_bf16(int *n) {
  static const Shape tab[] = {
      shape_of<bf16_t, Tout, 8, 16, 1>(), shape_of<bf16_t, Tout, 8, 32, 1>(), shape_of<bf16_t, Tout, 8, 64, 1>(),
      shape_of<bf16_t, Tout, 8, 64, 2>(), shape_of<bf16_t, Tout, 8, 64, 4>(), shape_of<bf16_t, Tout, 2, 64, 2>(),
      shape_of<bf16_t, Tout, 2, 64, 5>(),
  };
  *n = sizeof(tab) / sizeof(tab[0]);
  return tab;
}
template <typename Tout>
const Shape *shapes_f32(int *n) {
  static const Shape tab[] = {
      shape_of<float, Tout, 4, 16, 1>(), shape_of<float, Tout, 4, 32, 1>(), shape_of<float, Tout, 4, 64, 1>(),
      shape_of<float, Tout, 4, 64, 2>(), shape_of<float, Tout, 4, 64, 4>(), shape_of<float, Tout, 2, 64, 2>(),
      shape_of<float, Tout, 2, 64, 5>(), shape_of<float, Tout, 1, 64, 2>(), shape_of<float, Tout, 1, 64, 8>(),
  };
  *n = sizeof(tab) / sizeof(tab[0]);
  return tab;
}

}  // namespace

static const Shape *pick_shape(const SpmmArgs &a, int src_dtype, int out_dtype) {
  int n = 0;
  const Shape *tab;
  if (src_dtype == DT_BF16)
    tab = out_dtype == DT_BF16 ? shapes_bf16<bf16_t>(&n) : shapes_bf16<float>(&n);
  else
    tab = out_dtype == DT_BF16 ? shapes_f32<bf16_t>(&n) : shapes_f32<float>(&n);
  // widest vector that divides every leading dimension involved
  const bool has_aux = spmm_reads_aux(a.epilogue);
  const int lds[5] = {a.d, a.src_ld, a.out_ld, has_aux ? a.aux_ld : a.d, spmm_reads_add(a.epilogue) ? a.add_ld : a.d};
  const Shape *best = nullptr;
  int best_vec = 0;
  for (int i = 0; i < n; ++i) {
    bool ok = true;
    for (int k = 0; k < 5; ++k) ok = ok && (lds[k] % tab[i].vec == 0);
    if (ok && tab[i].vec > best_vec) best_vec = tab[i].vec;
  }
  if (best_vec == 0) return nullptr;  // bf16 rows of odd width are rejected at create time
  const int nvec = a.d / best_vec;
  for (int i = 0; i < n; ++i) {  // smallest tile that covers the row, else the widest tile
    if (tab[i].vec != best_vec) continue;
    const int cover = tab[i].lpr * tab[i].nv;
    if (best == nullptr) {
      best = &tab[i];
    } else {
      const int bc = best->lpr * best->nv;
      if ((bc < nvec && cover > bc) || (cover >= nvec && cover < bc)) best = &tab[i];
    }
  }
  return best;
}

static bool mfma_path(const SpmmArgs &a, int src_dtype) {
  const bool off = a.force_valu != 0;  // measurement switch
  const bool has_aux = spmm_reads_aux(a.epilogue);
  return !off && src_dtype == DT_BF16 && a.d % 8 == 0 && a.src_ld % 8 == 0 && a.out_ld % 8 == 0 &&
         (!has_aux || a.aux_ld % 8 == 0) && (!spmm_reads_add(a.epilogue) || a.add_ld % 8 == 0);
}

template <typename Tout, int NT>
static void launch_ring(const SpmmArgs &a, hipStream_t s, dim3 grid, int unroll) {
  const bool full = a.d == NT * 128;
  if (unroll >= 8) {
    if (full) hipLaunchKernelGGL((spmm_ring_kernel<Tout, NT, 8, true>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((spmm_ring_kernel<Tout, NT, 8, false>), grid, dim3(256), 0, s, a);
  } else if (unroll >= 4) {
    if (full) hipLaunchKernelGGL((spmm_ring_kernel<Tout, NT, 4, true>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((spmm_ring_kernel<Tout, NT, 4, false>), grid, dim3(256), 0, s, a);
  } else {
    if (full) hipLaunchKernelGGL((spmm_ring_kernel<Tout, NT, 2, true>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((spmm_ring_kernel<Tout, NT, 2, false>), grid, dim3(256), 0, s, a);
  }
}

template <typename Tout>
static int launch_mfma(const SpmmArgs &a_in, hipStream_t s) {
  SpmmArgs a = a_in;
  // short whole rows (the tail of the task list) are served a row per 16-lane group, by extra workgroups of the
  // same launch, when a row fits the registers of such a group
  const int64_t n_short = (a.d <= 256 && a.n_short > 0 && a.n_short <= a.n_tasks - a.tail_task0) ? a.n_short : 0;
  a.n_tasks -= n_short;
  a.n_short = n_short;
  a.n_main_blocks = a.n_class_blocks + (a.n_tasks - a.tail_task0 + 3) / 4;
  const unsigned gx = (unsigned)(a.n_main_blocks + (n_short + 15) / 16);
  if (gx == 0) return hipSuccess;  // only class pieces, none of them active
  const int unroll = a.unroll;  // 4 or 8 trade waves per SIMD for deeper per-wave queues (tests run all three)
  if (a.d <= 128)
    launch_ring<Tout, 1>(a, s, dim3(gx, 1), unroll);
  else if (a.d <= 256)
    launch_ring<Tout, 2>(a, s, dim3(gx, 1), unroll);
  else
    launch_ring<Tout, 4>(a, s, dim3(gx, (unsigned)((a.d + 511) / 512)), unroll >= 8 ? 4 : 2);
  return (int)hipGetLastError();
}

int launch_spmm(const SpmmArgs &a, int src_dtype, int out_dtype, hipStream_t s) {
  if (a.n_tasks <= 0) return hipSuccess;
  if (mfma_path(a, src_dtype)) return out_dtype == DT_BF16 ? launch_mfma<bf16_t>(a, s) : launch_mfma<float>(a, s);
  const Shape *best = pick_shape(a, src_dtype, out_dtype);
  if (!best) return hipErrorInvalidValue;
  const int tile_w = best->lpr * best->nv * best->vec;
  dim3 grid((unsigned)(a.n_class_blocks + (a.n_tasks - a.tail_task0 + 3) / 4), (unsigned)((a.d + tile_w - 1) / tile_w));
  if (grid.x == 0) return hipSuccess;
  hipLaunchKernelGGL(best->main, grid, dim3(256), 0, s, a);
  return (int)hipGetLastError();
}

int launch_spmm_reduce(const SpmmArgs &a, int src_dtype, int out_dtype, hipStream_t s) {
  if (a.n_long <= 0) return hipSuccess;
  const Shape *best = pick_shape(a, src_dtype, out_dtype);
  if (!best) return hipErrorInvalidValue;
  hipLaunchKernelGGL(best->reduce, dim3((unsigned)a.n_long), dim3(256), 0, s, a);
  return (int)hipGetLastError();
}
