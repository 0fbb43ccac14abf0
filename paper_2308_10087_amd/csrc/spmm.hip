// Neighbour aggregation with the current-vs-history select fused into the gather
// (Algorithm 1, the AGGREGATE line; Section 3.3), and its transposed twin for the
// backward pass where unselected entries contribute zero (Section 3.4, technique 3).
//
// One wavefront per task.  A task is a whole sparse row, or a piece of a long row (power-law
// hubs are cut so that no wave owns more than a fixed number of entries; the pieces write
// fp32 partial sums that a second small kernel adds in a fixed order, so results do not
// depend on scheduling).  Inside a wave the 64 lanes form G = 64/LPR groups of LPR lanes;
// each group gathers one neighbour row per step with 16-byte loads (LPR * 16 B covers the
// row), so a 512-byte bf16 row of width 256 is one half-wave load and two neighbours are in
// flight per instruction.  Entry metadata (packed index, weight) is loaded 64 entries at a
// time, one per lane, and broadcast through lane permutes; when unselected entries are
// dropped they are first compacted inside the wave so that no bandwidth is spent on them.
#include <stdlib.h>

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

// Applies the epilogue to VEC consecutive columns of one output row and stores them.
template <typename Tin, typename Tout, int VEC>
__device__ inline void finish_cols(const SpmmArgs &a, int64_t row, int c, const float (&acc)[VEC]) {
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
  } else {
    const Pack<Tin, VEC> x = *reinterpret_cast<const Pack<Tin, VEC> *>(
        static_cast<const Tin *>(a.aux) + (size_t)row * a.aux_ld + c);
    if (a.epilogue == SPMM_MIX) {
#pragma unroll
      for (int t = 0; t < VEC; ++t) r[t] = a.s_acc * acc[t] + a.s_aux * to_f32(x.v[t]);
    } else {
#pragma unroll
      for (int t = 0; t < VEC; ++t) r[t] = to_f32(x.v[t]) > 0.f ? acc[t] : 0.f;
    }
  }
  Pack<Tout, VEC> o;
#pragma unroll
  for (int t = 0; t < VEC; ++t) o.v[t] = from_f32<Tout>(r[t]);
  *reinterpret_cast<Pack<Tout, VEC> *>(static_cast<Tout *>(a.out) + (size_t)(row - a.out_row0) * a.out_ld + c) = o;
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
template <typename Tin, typename Tout, int VEC>
__global__ __launch_bounds__(256) void spmm_reduce_kernel(const SpmmArgs a) {
  __shared__ float red[8][32][VEC];
  const int64_t i = blockIdx.x;
  const int ph = threadIdx.x >> 5, cv = threadIdx.x & 31;
  const int64_t row = a.lr_row[i];
  const int slot0 = a.lr_slot0[i], ns = a.lr_nslots[i];
  // pieces of classes that were not run in this launch (all their entries unselected) hold stale data
  const bool check = a.slot_class != nullptr && a.all_classes_active == 0;
  for (int c0 = 0; c0 < a.d; c0 += 32 * VEC) {
    const int c = c0 + cv * VEC;
    float acc[VEC];
#pragma unroll
    for (int t = 0; t < VEC; ++t) acc[t] = 0.f;
    if (c < a.d) {
      for (int s = ph; s < ns; s += 8) {
        if (check) {
          const uint32_t sc = a.slot_class[slot0 + s];
          if (sc < 32u && !((a.active_classes >> sc) & 1u)) continue;
        }
        const Pack<float, VEC> x = *reinterpret_cast<const Pack<float, VEC> *>(a.partial + (size_t)(slot0 + s) * a.d + c);
#pragma unroll
        for (int t = 0; t < VEC; ++t) acc[t] += x.v[t];
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
      finish_cols<Tin, Tout, VEC>(a, row, c, acc);
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

template <typename Tout, int NT, int U>
__global__ __launch_bounds__(256) void spmm_mfma_kernel(const SpmmArgs a) {
  constexpr int TILE_W = NT * 128;
  __shared__ float rowbuf[4][TILE_W];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t task = spmm_task_index(a, blockIdx.x, wave);
  if (task < 0) return;  // whole wave leaves together (no block-wide barrier below)
  const int g = lane >> 4, lig = lane & 15;
  const int tile0 = blockIdx.y * TILE_W;
  // task fields are the same for the whole wave: keep them in scalar registers.  The matrix
  // instruction ignores the execution mask and the lane permutes need every lane in step, so all
  // control flow around them must be provably wave-uniform.
  const int64_t row = __builtin_amdgcn_readfirstlane(a.task_row[task]);
  const int64_t e0_raw = a.task_e0[task];
  const int64_t e0 = ((int64_t)__builtin_amdgcn_readfirstlane((int)(e0_raw >> 32)) << 32) |
                     (uint32_t)__builtin_amdgcn_readfirstlane((int)(e0_raw & 0xffffffff));
  const int ne = __builtin_amdgcn_readfirstlane(a.task_ne[task]);
  const int slot = __builtin_amdgcn_readfirstlane(a.task_slot[task]);
  const uint32_t vmask = (1u << a.vbits) - 1u;
  const bool drop_unsel = a.src_unsel == nullptr;
  const bf16_t *src_sel = static_cast<const bf16_t *>(a.src_sel);
  const bf16_t *src_unsel = static_cast<const bf16_t *>(a.src_unsel);
  const int d = a.d;
  const size_t ld = (size_t)a.src_ld;
  const int pos = lig & 7;            // which element of the 8-column block this lane's B column picks
  const bool lo_part = lig >= 8;      // B columns 8..15 carry the low half of the weight

  f32x4_t acc[NT];
#pragma unroll
  for (int h = 0; h < NT; ++h) acc[h] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  const bf16x8_t zero8 = {0, 0, 0, 0, 0, 0, 0, 0};

  // entry metadata of the first batch; later batches are fetched one batch ahead
  uint32_t pc_next = 0;
  float w_next = 0.f;
  if (lane < ne) {
    pc_next = a.pidx[e0 + lane];
    w_next = a.val[e0 + lane];
  }
  for (int base = 0; base < ne; base += 64) {
    int n = ne - base < 64 ? ne - base : 64;
    const uint32_t pc = pc_next;
    float w = w_next;
    if (base + 64 + lane < ne) {
      pc_next = a.pidx[e0 + base + 64 + lane];
      w_next = a.val[e0 + base + 64 + lane];
    }
    uint32_t info = 0;
    bool keep = false;
    if (lane < n) {
      const bool sel = mask_test(a.mask, pc >> a.vbits);
      keep = sel || !drop_unsel;
      info = (pc & vmask) | (sel ? 0x80000000u : 0u);
    } else {
      w = 0.f;
    }
    if (drop_unsel) {
      const uint64_t bal = __ballot(keep);
      const int nk = __popcll(bal);
      const int rk = __popcll(bal & ((1ull << lane) - 1ull));
      const int dest = keep ? rk : nk + (lane - rk);
      info = (uint32_t)__builtin_amdgcn_ds_permute(dest << 2, (int)info);
      w = __int_as_float(__builtin_amdgcn_ds_permute(dest << 2, __float_as_int(w)));
      n = __builtin_amdgcn_readfirstlane(nk);
    }
    // U*4 entries per step: all gathers of the step are issued before the first product needs its data.
    // What bounds this kernel is the number of bytes in flight per compute unit, i.e. the share of the
    // register file that holds gathered rows: a step keeps U*NT 16-byte pieces per lane pending, and the
    // weight operand is kept as one packed word per neighbour and expanded only when it is multiplied.
    for (int i = 0; i < n; i += 4 * U) {
      bf16x8_t x[U][NT];
      uint32_t wbits[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (i + 4 * u < n) {  // wave-uniform
          const int idx = i + 4 * u + g;
          const int from = idx < n ? idx : i;  // past the end: a valid row with weight 0
          const uint32_t inf = (uint32_t)__shfl((int)info, from);
          float ww = __shfl(w, from);
          if (idx >= n) ww = 0.f;
          // split the fp32 weight into two bf16 halves; this lane's half goes to element `pos` of B
          const bf16_t whi = (bf16_t)ww;
          const bf16_t wlo = (bf16_t)(ww - (float)whi);
          const bf16_t part = lo_part ? wlo : whi;
          wbits[u] = (uint32_t)__builtin_bit_cast(uint16_t, part) << ((pos & 1) * 16);
          const bf16_t *rowp = ((inf >> 31) ? src_sel : src_unsel) + (size_t)(inf & 0x7fffffffu) * ld + tile0 + lig * 8;
#pragma unroll
          for (int h = 0; h < NT; ++h)
            x[u][h] = (tile0 + h * 128 + lig * 8 < d) ? *reinterpret_cast<const bf16x8_t *>(rowp + h * 128) : zero8;
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (i + 4 * u < n) {
          u32x4_t bw;
          bw[0] = (pos >> 1) == 0 ? wbits[u] : 0u;
          bw[1] = (pos >> 1) == 1 ? wbits[u] : 0u;
          bw[2] = (pos >> 1) == 2 ? wbits[u] : 0u;
          bw[3] = (pos >> 1) == 3 ? wbits[u] : 0u;
          const bf16x8_t bfrag = __builtin_bit_cast(bf16x8_t, bw);
#pragma unroll
          for (int h = 0; h < NT; ++h) acc[h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x[u][h], bfrag, acc[h], 0, 0, 0);
        }
      }
    }
  }
  // D layout: element i of lane l is D[m = 4*(l/16) + i][n = l%16]; column = 8m + n%8, halves n<8 / n>=8
#pragma unroll
  for (int h = 0; h < NT; ++h)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float v = acc[h][i] + __shfl_xor(acc[h][i], 8);
      if (!lo_part) rowbuf[wave][h * 128 + (4 * g + i) * 8 + pos] = v;
    }
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the wave's own LDS writes have landed
  // natural layout again: lane q owns 8 consecutive columns
#pragma unroll
  for (int r = 0; r < (NT * 16 + 63) / 64; ++r) {
    const int q = lane + 64 * r;
    const int c = tile0 + q * 8;
    if (q < NT * 16 && c < d) {
      float v[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) v[t] = rowbuf[wave][q * 8 + t];
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
  const bool has_aux = a.epilogue == SPMM_MIX || a.epilogue == SPMM_MASK;
  const int lds[4] = {a.d, a.src_ld, a.out_ld, has_aux ? a.aux_ld : a.d};
  const Shape *best = nullptr;
  int best_vec = 0;
  for (int i = 0; i < n; ++i) {
    bool ok = true;
    for (int k = 0; k < 4; ++k) ok = ok && (lds[k] % tab[i].vec == 0);
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
  static const bool off = getenv("GNNSTAGE_SPMM_VALU") != nullptr;  // measurement switch
  const bool has_aux = a.epilogue == SPMM_MIX || a.epilogue == SPMM_MASK;
  return !off && src_dtype == DT_BF16 && a.d % 8 == 0 && a.src_ld % 8 == 0 && a.out_ld % 8 == 0 &&
         (!has_aux || a.aux_ld % 8 == 0);
}

template <typename Tout>
static int launch_mfma(const SpmmArgs &a, hipStream_t s) {
  const unsigned gx = (unsigned)(a.n_class_blocks + (a.n_tasks - a.tail_task0 + 3) / 4);
  if (gx == 0) return hipSuccess;  // only class pieces, none of them active
  static const int unroll = getenv("GNNSTAGE_SPMM_UNROLL") ? atoi(getenv("GNNSTAGE_SPMM_UNROLL")) : 4;
  if (a.d <= 128) {
    if (unroll >= 8)
      hipLaunchKernelGGL((spmm_mfma_kernel<Tout, 1, 8>), dim3(gx, 1), dim3(256), 0, s, a);
    else if (unroll >= 4)
      hipLaunchKernelGGL((spmm_mfma_kernel<Tout, 1, 4>), dim3(gx, 1), dim3(256), 0, s, a);
    else
      hipLaunchKernelGGL((spmm_mfma_kernel<Tout, 1, 2>), dim3(gx, 1), dim3(256), 0, s, a);
  } else if (a.d <= 256) {
    if (unroll >= 4)
      hipLaunchKernelGGL((spmm_mfma_kernel<Tout, 2, 4>), dim3(gx, 1), dim3(256), 0, s, a);
    else
      hipLaunchKernelGGL((spmm_mfma_kernel<Tout, 2, 2>), dim3(gx, 1), dim3(256), 0, s, a);
  } else {
    hipLaunchKernelGGL((spmm_mfma_kernel<Tout, 4, 4>), dim3(gx, (unsigned)((a.d + 511) / 512)), dim3(256), 0, s, a);
  }
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
