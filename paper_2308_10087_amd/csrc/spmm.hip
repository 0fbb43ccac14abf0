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
  const int64_t task = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (task >= a.n_tasks) return;  // whole wave leaves together
  const int grp = lane / LPR, lig = lane % LPR;
  const int col0 = blockIdx.y * TILE_W + lig * VEC;
  const int64_t row = a.task_row[task];
  const int64_t e0 = a.task_e0[task];
  const int ne = a.task_ne[task];
  const int slot = a.task_slot[task];
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
      n = nk;
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

// Sums the pieces of every long row in slot order, then applies the epilogue.
template <typename Tin, typename Tout, int VEC>
__global__ __launch_bounds__(256) void spmm_reduce_kernel(const SpmmArgs a) {
  const int64_t i = blockIdx.x;
  const int64_t row = a.lr_row[i];
  const int slot0 = a.lr_slot0[i], ns = a.lr_nslots[i];
  for (int c = threadIdx.x * VEC; c < a.d; c += blockDim.x * VEC) {
    float acc[VEC];
#pragma unroll
    for (int t = 0; t < VEC; ++t) acc[t] = 0.f;
    for (int s = 0; s < ns; ++s) {
      const Pack<float, VEC> x = *reinterpret_cast<const Pack<float, VEC> *>(a.partial + (size_t)(slot0 + s) * a.d + c);
#pragma unroll
      for (int t = 0; t < VEC; ++t) acc[t] += x.v[t];
    }
    finish_cols<Tin, Tout, VEC>(a, row, c, acc);
  }
  if (threadIdx.x < 64) zero_pad_cols<Tout>(a, row, threadIdx.x);
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

int launch_spmm(const SpmmArgs &a, int src_dtype, int out_dtype, hipStream_t s) {
  if (a.n_tasks <= 0) return hipSuccess;
  const Shape *best = pick_shape(a, src_dtype, out_dtype);
  if (!best) return hipErrorInvalidValue;
  const int tile_w = best->lpr * best->nv * best->vec;
  dim3 grid((unsigned)((a.n_tasks + 3) / 4), (unsigned)((a.d + tile_w - 1) / tile_w));
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
