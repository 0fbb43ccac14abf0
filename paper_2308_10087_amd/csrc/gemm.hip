// Dense transforms of the stage (the UPDATE line of Algorithm 1 and its gradients).
//
//   NT:  C[M x N]  = A[M x K] . Bt[N x Kp]^T      forward transform and input gradient
//   TN:  dW[I x O] += s * A[M x I]^T . B[M x O]    weight gradient (reduction over chunk rows)
//
// bf16 operands go through the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32
// accumulation); the fp32 variants are plain LDS-tiled FMA kernels used by the fp32 stage.
// Bias / ReLU / GCNII residual terms are applied in the epilogue on the fp32 accumulators.
// Bt and B always live in the library's zero-padded internal buffers (16-byte aligned rows);
// A may also be a caller-owned level buffer of any width and of fp32 or bf16 type, in which case
// it is read element-wise with bounds checks and converted while it is staged into LDS.
#include <stdlib.h>

#include "common.h"

namespace {

typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef bf16_t bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ inline float to_f32(float x) { return x; }
__device__ inline float to_f32(bf16_t x) { return (float)x; }

__device__ inline float load_f32(const void *p, int dtype, size_t idx) {
  return dtype == DT_BF16 ? (float)static_cast<const bf16_t *>(p)[idx] : static_cast<const float *>(p)[idx];
}
__device__ inline void store_f32(void *p, int dtype, size_t idx, float v) {
  if (dtype == DT_BF16)
    static_cast<bf16_t *>(p)[idx] = (bf16_t)v;
  else
    static_cast<float *>(p)[idx] = v;
}

// One output element of an NT product: epilogue + store.
__device__ inline void epilogue_store(const GemmNtArgs &a, int m, int n, float acc) {
  float r;
  switch (a.epilogue) {
    case EPI_FWD_GCN: {
      r = acc + a.bias[n];
      r = r > 0.f ? r : 0.f;
      break;
    }
    case EPI_FWD_GCNII: {
      const float p = load_f32(a.aux, a.aux_dtype, (size_t)m * a.aux_ld + n);
      r = (1.f - a.beta) * p + a.beta * acc;
      r = r > 0.f ? r : 0.f;
      break;
    }
    case EPI_PLAIN: {
      r = acc;
      break;
    }
    case EPI_FWD_ADD: {
      r = acc + a.bias[n] + load_f32(a.aux, a.aux_dtype, (size_t)m * a.aux_ld + n);
      r = r > 0.f ? r : 0.f;
      break;
    }
    case EPI_RES: {
      r = acc + a.bias[n] + load_f32(a.aux, a.aux_dtype, (size_t)m * a.aux_ld + n);
      break;
    }
    case EPI_MASK: {
      r = load_f32(a.aux, a.aux_dtype, (size_t)m * a.aux_ld + n) > 0.f ? acc * a.mask_scale : 0.f;
      break;
    }
    default: {  // EPI_DGRAD_GCNII
      const float dy = load_f32(a.aux, a.aux_dtype, (size_t)m * a.aux_ld + n);
      const float dp = (1.f - a.beta) * dy + a.beta * acc;
      r = (1.f - a.alpha) * dp;
      if (a.h0grad) a.h0grad[(size_t)m * a.h0_ld + n] += a.alpha * dp;
      break;
    }
  }
  store_f32(a.out, a.out_dtype, (size_t)m * a.out_ld + n, r);
}

__device__ inline void load8_f32(const void *p, int dtype, size_t idx, float (&v)[8]) {
  if (dtype == DT_BF16) {
    const bf16x8 x = *reinterpret_cast<const bf16x8 *>(static_cast<const bf16_t *>(p) + idx);
#pragma unroll
    for (int t = 0; t < 8; ++t) v[t] = (float)x[t];
  } else {
    const f32x4 x0 = *reinterpret_cast<const f32x4 *>(static_cast<const float *>(p) + idx);
    const f32x4 x1 = *reinterpret_cast<const f32x4 *>(static_cast<const float *>(p) + idx + 4);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      v[t] = x0[t];
      v[4 + t] = x1[t];
    }
  }
}
__device__ inline void store8_f32(void *p, int dtype, size_t idx, const float (&v)[8]) {
  if (dtype == DT_BF16) {
    bf16x8 x;
#pragma unroll
    for (int t = 0; t < 8; ++t) x[t] = (bf16_t)v[t];
    *reinterpret_cast<bf16x8 *>(static_cast<bf16_t *>(p) + idx) = x;
  } else {
    f32x4 x0, x1;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      x0[t] = v[t];
      x1[t] = v[4 + t];
    }
    *reinterpret_cast<f32x4 *>(static_cast<float *>(p) + idx) = x0;
    *reinterpret_cast<f32x4 *>(static_cast<float *>(p) + idx + 4) = x1;
  }
}

// Eight consecutive output columns n0..n0+7 of row m (all inside [0, N), every pointer involved
// 16-byte aligned at that position: checked on the host, a.vec_epi).
// epi: the epilogue to apply (a.epilogue, or EPI_PLAIN where the caller has applied it to the accumulators already)
__device__ inline void epilogue_store8(const GemmNtArgs &a, int m, int n0, const float (&acc)[8], int epi) {
  float r[8], x[8];
  switch (epi) {
    case EPI_FWD_GCN: {
      load8_f32(a.bias, DT_F32, (size_t)n0, x);
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const float y = acc[t] + x[t];
        r[t] = y > 0.f ? y : 0.f;
      }
      break;
    }
    case EPI_FWD_GCNII: {
      load8_f32(a.aux, a.aux_dtype, (size_t)m * a.aux_ld + n0, x);
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const float y = (1.f - a.beta) * x[t] + a.beta * acc[t];
        r[t] = y > 0.f ? y : 0.f;
      }
      break;
    }
    case EPI_PLAIN: {
#pragma unroll
      for (int t = 0; t < 8; ++t) r[t] = acc[t];
      break;
    }
    case EPI_FWD_ADD:
    case EPI_RES: {
      float b8[8];
      load8_f32(a.bias, DT_F32, (size_t)n0, b8);
      load8_f32(a.aux, a.aux_dtype, (size_t)m * a.aux_ld + n0, x);
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const float y = acc[t] + b8[t] + x[t];
        r[t] = (epi == EPI_RES || y > 0.f) ? y : 0.f;
      }
      break;
    }
    case EPI_MASK: {
      load8_f32(a.aux, a.aux_dtype, (size_t)m * a.aux_ld + n0, x);
#pragma unroll
      for (int t = 0; t < 8; ++t) r[t] = x[t] > 0.f ? acc[t] * a.mask_scale : 0.f;
      break;
    }
    default: {  // EPI_DGRAD_GCNII
      load8_f32(a.aux, a.aux_dtype, (size_t)m * a.aux_ld + n0, x);
      float dp[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        dp[t] = (1.f - a.beta) * x[t] + a.beta * acc[t];
        r[t] = (1.f - a.alpha) * dp[t];
      }
      if (a.h0grad) {
        float h[8];
        load8_f32(a.h0grad, DT_F32, (size_t)m * a.h0_ld + n0, h);
#pragma unroll
        for (int t = 0; t < 8; ++t) h[t] += a.alpha * dp[t];
        store8_f32(a.h0grad, DT_F32, (size_t)m * a.h0_ld + n0, h);
      }
      break;
    }
  }
  store8_f32(a.out, a.out_dtype, (size_t)m * a.out_ld + n0, r);
}

// 8 consecutive elements of row `r` starting at column `c` as bf16; columns >= cols read as zero.
template <typename T, bool VEC>
__device__ inline bf16x8 load8_bf16(const T *base, size_t ld, int r, int c, int cols) {
  bf16x8 out = {0, 0, 0, 0, 0, 0, 0, 0};
  if constexpr (VEC) {
    if (c < cols) out = *reinterpret_cast<const bf16x8 *>(base + (size_t)r * ld + c);
  } else {
    const T *p = base + (size_t)r * ld + c;
#pragma unroll
    for (int t = 0; t < 8; ++t)
      if (c + t < cols) out[t] = (bf16_t)to_f32(p[t]);
  }
  return out;
}

// ------------------------------------------------------------------------------------ bf16 NT
constexpr int BM = 128, BN = 128;
// K step BK = 32 or 64 elements per LDS tile; rows are padded by 8 elements (80- or 144-byte rows keep the 16-byte
// fragment reads conflict-free).  The per-chunk products of small graphs (a few ten thousand rows: one or two
// workgroups per CU, all resident at once) are a chain of K / BK load-wait-multiply steps and nothing else, so the
// deeper step halves their time's main term; it costs registers (four staged vectors per operand) and LDS (72 KB
// per workgroup), which the long products do not have to spare.

// PAIR: A is an fp32 matrix with an even leading dimension and an 8-byte aligned base.  A tile row is then
// 32 floats = one 128-byte line, read by 16 lanes as float pairs (four whole rows per wave instruction,
// fully coalesced) instead of eight scalars per lane.
template <typename TA, bool VEC, bool PAIR = false, int BK = 32>
__global__ __launch_bounds__(256) void gemm_nt_bf16_kernel(const GemmNtArgs a) {
  constexpr int LDS_K = BK + 8;   // padded K stride (elements)
  constexpr int KV = BK / 8;      // 16-byte vectors per tile row
  constexpr int NV = BM * KV / 256;  // vectors per thread and operand tile
  static_assert(!PAIR || BK == 32, "the float-pair loader is written for 32-wide steps");
  __shared__ __attribute__((aligned(16))) bf16_t As[2][BM * LDS_K];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[2][BN * LDS_K];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  // Workgroups go round-robin over the 8 XCDs (each with its own L2).  The column tiles that share a
  // block of A rows are given consecutive slots on ONE XCD, so A is fetched into that L2 once.
  const int nt = (a.N + BN - 1) / BN;
  const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
  const int m0 = ((q / nt) * 8 + xcd) * BM, n0 = (q % nt) * BN;
  if (m0 >= a.M) return;  // padding slots of the last group of 8 row tiles
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
  const TA *A = static_cast<const TA *>(a.A);
  const bf16_t *Bt = static_cast<const bf16_t *>(a.Bt);
  const int a_cols = VEC ? a.Kp : a.K;  // padded operands are valid (zero) up to Kp

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int t = 0; t < 16; ++t) acc[i][j][t] = 0.f;

  bf16x8 ra[NV], rb[NV];
  f32x2 rp[PAIR ? 8 : 1];
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  auto gload = [&](int k0) {
    if constexpr (PAIR) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int r = (tid >> 4) + 16 * i, k = k0 + 2 * (tid & 15);
        f32x2 v = {0.f, 0.f};
        if (m0 + r < a.M) {
          const float *p = reinterpret_cast<const float *>(A) + (size_t)(m0 + r) * a.lda + k;
          if (k + 1 < a.K)
            v = *reinterpret_cast<const f32x2 *>(p);
          else if (k < a.K)
            v[0] = p[0];
        }
        rp[i] = v;
      }
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int vid = tid + 256 * i, r = vid / KV, k = k0 + (vid % KV) * 8;
      if constexpr (!PAIR) ra[i] = (m0 + r < a.M) ? load8_bf16<TA, VEC>(A, (size_t)a.lda, m0 + r, k, a_cols) : zero8;
      rb[i] = (n0 + r < a.N && k < a.Kp) ? *reinterpret_cast<const bf16x8 *>(Bt + (size_t)(n0 + r) * a.ldb + k) : zero8;
    }
  };
  auto sstore = [&](int buf) {
    if constexpr (PAIR) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int r = (tid >> 4) + 16 * i;
        const bf16x2 v = {(bf16_t)rp[i][0], (bf16_t)rp[i][1]};
        *reinterpret_cast<bf16x2 *>(&As[buf][r * LDS_K + 2 * (tid & 15)]) = v;
      }
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int vid = tid + 256 * i, r = vid / KV, kv = vid % KV;
      if constexpr (!PAIR) *reinterpret_cast<bf16x8 *>(&As[buf][r * LDS_K + kv * 8]) = ra[i];
      *reinterpret_cast<bf16x8 *>(&Bs[buf][r * LDS_K + kv * 8]) = rb[i];
    }
  };

  const int nk = (a.Kp + BK - 1) / BK;
  gload(0);
  sstore(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) gload((kt + 1) * BK);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 fa[2], fb[2];
      const int koff = kk * 16 + (lane >> 5) * 8;
#pragma unroll
      for (int i = 0; i < 2; ++i)
        fa[i] = *reinterpret_cast<const bf16x8 *>(&As[buf][(wm + i * 32 + (lane & 31)) * LDS_K + koff]);
#pragma unroll
      for (int j = 0; j < 2; ++j)
        fb[j] = *reinterpret_cast<const bf16x8 *>(&Bs[buf][(wn + j * 32 + (lane & 31)) * LDS_K + koff]);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) {
      sstore(buf ^ 1);  // the other buffer was last read before the previous barrier
      __syncthreads();
    }
  }
  // 32x32 accumulator layout: element t of lane l is row 8*(t/4) + 4*(l/32) + t%4, column l%32.
  // Each wave passes its tiles through a private LDS patch so that a lane ends up with 8 consecutive
  // columns of one row: 16-byte stores and vector reads of bias / residual rows.
  __syncthreads();  // every wave is done with the operand tiles; As is reused as staging space
  constexpr int PS = 36;  // padded row stride (floats) of the 32x32 patch
  float *patch = reinterpret_cast<float *>(&As[0][0]) + wave * (32 * PS);
  static_assert(4 * 32 * PS * sizeof(float) <= sizeof(As), "staging patch must fit the A tiles");
  // GCN forward epilogue: bias + ReLU on the accumulators, where a lane holds one column of a sub-tile (two bias
  // values per lane), instead of a bias load in front of each of the lane's eight row-wise pieces
  const bool gcn_fwd = a.vec_epi && a.epilogue == EPI_FWD_GCN;
  float bias_col[2] = {0.f, 0.f};
  if (gcn_fwd) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int n = n0 + wn + j * 32 + (lane & 31);
      if (n < a.N) bias_col[j] = a.bias[n];
    }
  }
  const int store_epi = gcn_fwd ? (int)EPI_PLAIN : (int)a.epilogue;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int mt = m0 + wm + i * 32, nt = n0 + wn + j * 32;
      if (mt >= a.M || nt >= (a.out_pad > a.N ? a.out_pad : a.N)) continue;  // wave-uniform
      if (a.vec_epi) {
        if (gcn_fwd) {
#pragma unroll
          for (int t = 0; t < 16; ++t) {
            const float y = acc[i][j][t] + bias_col[j];
            acc[i][j][t] = y > 0.f ? y : 0.f;
          }
        }
#pragma unroll
        for (int t = 0; t < 16; ++t) patch[(8 * (t >> 2) + 4 * (lane >> 5) + (t & 3)) * PS + (lane & 31)] = acc[i][j][t];
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int ps = 0; ps < 2; ++ps) {
          const int idx = ps * 64 + lane, r = idx >> 2, c = (idx & 3) * 8;
          float v[8];
          const f32x4 v0 = *reinterpret_cast<const f32x4 *>(&patch[r * PS + c]);
          const f32x4 v1 = *reinterpret_cast<const f32x4 *>(&patch[r * PS + c + 4]);
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            v[t] = v0[t];
            v[4 + t] = v1[t];
          }
          if (mt + r < a.M && nt + c < a.N) epilogue_store8(a, mt + r, nt + c, v, store_epi);
        }
        __builtin_amdgcn_wave_barrier();
      } else {
#pragma unroll
        for (int t = 0; t < 16; ++t) {
          const int m = mt + 8 * (t >> 2) + 4 * (lane >> 5) + (t & 3);
          const int n = nt + (lane & 31);
          if (m < a.M && n < a.N)
            epilogue_store(a, m, n, acc[i][j][t]);
          else if (m < a.M && n < a.out_pad)
            store_f32(a.out, a.out_dtype, (size_t)m * a.out_ld + n, 0.f);
        }
      }
    }
}

// ------------------------------------------------------------- bf16 NT, weight-stationary and persistent
// For the widths of this stage (K, N <= 256) the product streams A in and C out and is HBM-bound; what
// decides its speed is how many bytes of A are in flight, not arithmetic.  Each wave keeps its 64-column
// panel of Bt in registers for the whole kernel (as ready-made MFMA fragments), workgroups are persistent
// and walk over row tiles, and the loads of the next A tile are in flight while the current one is
// multiplied and stored.  WN = column panels per workgroup (4: N <= 256 with 64-row tiles, 2: N <= 128
// with 128-row tiles); KS = number of 16-wide k-steps held (Kp <= 16 * KS).
// GCNF: the instance for the GCN forward epilogue (bias + ReLU applied to the accumulators, see below).
template <int WN, int KS, bool GCNF>
__global__ __launch_bounds__(256, 2) void gemm_nt_bf16_ws_kernel(const GemmNtArgs a) {
  constexpr int WR = 4 / WN, TM = 64 * WR;  // row groups, rows per tile
  constexpr int LDK = KS * 16 + 8;          // LDS row stride (elements): conflict-free 16-byte fragment reads
  constexpr int NV = TM * (KS * 2) / 256;   // 16-byte vectors of an A tile per thread
  constexpr int PS = 40;                    // padded row stride (floats) of a 16x32 staging patch
  constexpr int PB = 40;                    // padded row stride (bf16) of the 32x32 patch of the plain bf16 store
  static_assert(32 * PB * sizeof(bf16_t) <= 16 * PS * sizeof(float), "the bf16 patch reuses the fp32 patch's memory");
  extern __shared__ __attribute__((aligned(16))) unsigned char ws_smem[];
  bf16_t *As = reinterpret_cast<bf16_t *>(ws_smem);                                 // [2][TM * LDK]
  float *patches = reinterpret_cast<float *>(ws_smem + (size_t)2 * TM * LDK * 2);  // [4][16 * PS]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int rg = wave / WN, cp = wave % WN;
  const bf16_t *A = static_cast<const bf16_t *>(a.A);
  const bf16_t *Bt = static_cast<const bf16_t *>(a.Bt);
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  const int kl = (lane >> 5) * 8;
  const int n_wave = cp * 64;

  // this wave's panel of Bt as MFMA B fragments: [k-step][column sub-tile]
  bf16x8 bfr[KS][2];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int n = n_wave + j * 32 + (lane & 31), k = ks * 16 + kl;
      bfr[ks][j] = (n < a.N && k < a.Kp) ? *reinterpret_cast<const bf16x8 *>(Bt + (size_t)n * a.ldb + k) : zero8;
    }

  // GCN forward epilogue (bias + ReLU): in the accumulator layout a lane holds ONE column of a 32 x 32 sub-tile, so
  // the bias is two values per lane for the whole kernel, added (and clamped) before the sub-tile goes through the
  // LDS patch; the store that follows is the plain one.  Loading the bias piece by piece in the row-wise layout after
  // the patch cost a dependent load per piece: 11.2 against 9.5 ms per c4 step for the forward products.
  // An instance of its own, so that the other epilogues do not carry its registers (with one kernel for both, the plain
  // input-gradient products went from 7.0 to 7.5 ms per c4 step).
  constexpr bool gcn_fwd = GCNF;
  float bias_col[2] = {0.f, 0.f};
  if constexpr (gcn_fwd) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int n = n_wave + j * 32 + (lane & 31);
      if (n < a.N) bias_col[j] = a.bias[n];
    }
  }
  const int store_epi = gcn_fwd ? (int)EPI_PLAIN : (int)a.epilogue;  // what the store path still has to apply
  // Plain bf16 stores (the GCN forward product after the lines above, the GCN input-gradient product): the sub-tile is
  // rounded to bf16 in the accumulator layout and passes through LDS whole, as 2-byte elements; a lane then reads and
  // stores two 16-byte row pieces.  Half as many write - wait - read round trips per tile as the general path below,
  // which was the largest part of a tile's time (clock reads in an instrumented build: of 5.2 us per 64-row tile 1.75
  // were the matrix chains, 2.8 the stores, 0.7 barriers and staging).
  const bool plain_bf16 = a.vec_epi && store_epi == EPI_PLAIN && a.out_dtype == DT_BF16;
  const int n_tiles = (a.M + TM - 1) / TM;
  bf16x8 stage[NV];
  auto gload = [&](int tile) {
    const int m0 = tile * TM;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int vid = tid + 256 * i, r = vid / (KS * 2), k = (vid % (KS * 2)) * 8;
      stage[i] = (m0 + r < a.M && k < a.Kp) ? *reinterpret_cast<const bf16x8 *>(A + (size_t)(m0 + r) * a.lda + k) : zero8;
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int vid = tid + 256 * i, r = vid / (KS * 2), k = (vid % (KS * 2)) * 8;
      *reinterpret_cast<bf16x8 *>(&As[buf * TM * LDK + r * LDK + k]) = stage[i];
    }
  };

  int tile = blockIdx.x;
  if (tile >= n_tiles) return;
  gload(tile);
  sstore(0);
  __syncthreads();
  float *patch = patches + wave * (16 * PS);
  int buf = 0;
  for (; tile < n_tiles; tile += gridDim.x, buf ^= 1) {
    const int next = tile + gridDim.x;
    if (next < n_tiles) gload(next);  // in flight during the products and the stores below
    const bf16_t *At = As + buf * TM * LDK + (rg * 64) * LDK;
    const int m_wave = tile * TM + rg * 64;
    // the wave's 64x64 block, one 32x32 sub-tile at a time (few accumulator registers: the Bt panel
    // already takes KS*8), each written out through the wave's private LDS patch in two 16-row halves
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        f32x16 acc;
#pragma unroll
        for (int t = 0; t < 16; ++t) acc[t] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const bf16x8 fa = *reinterpret_cast<const bf16x8 *>(&At[(i * 32 + (lane & 31)) * LDK + ks * 16 + kl]);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, bfr[ks][j], acc, 0, 0, 0);
        }
        const int mt = m_wave + i * 32, ntc = n_wave + j * 32;
        if (mt >= a.M || ntc >= (a.out_pad > a.N ? a.out_pad : a.N)) continue;  // wave-uniform
        if (a.vec_epi) {
          if constexpr (gcn_fwd) {
#pragma unroll
            for (int t = 0; t < 16; ++t) {
              const float y = acc[t] + bias_col[j];
              acc[t] = y > 0.f ? y : 0.f;
            }
          }
          if (plain_bf16) {
            bf16_t *bp = reinterpret_cast<bf16_t *>(patch);
#pragma unroll
            for (int t = 0; t < 16; ++t) bp[(8 * (t >> 2) + 4 * (lane >> 5) + (t & 3)) * PB + (lane & 31)] = (bf16_t)acc[t];
            __builtin_amdgcn_wave_barrier();
            bf16_t *outp = static_cast<bf16_t *>(a.out);
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
              const int r = (lane >> 2) + 16 * hf, c = (lane & 3) * 8;
              const bf16x8 v = *reinterpret_cast<const bf16x8 *>(&bp[r * PB + c]);
              if (mt + r < a.M && ntc + c < a.N) *reinterpret_cast<bf16x8 *>(outp + (size_t)(mt + r) * a.out_ld + ntc + c) = v;
            }
            __builtin_amdgcn_wave_barrier();
            continue;
          }
#pragma unroll
          for (int hf = 0; hf < 2; ++hf) {  // accumulator elements 8*hf .. 8*hf+7 are rows 16*hf .. 16*hf+15
#pragma unroll
            for (int t = 0; t < 8; ++t)
              patch[(8 * (t >> 2) + 4 * (lane >> 5) + (t & 3)) * PS + (lane & 31)] = acc[8 * hf + t];
            __builtin_amdgcn_wave_barrier();
            const int r = lane >> 2, c = (lane & 3) * 8;
            float v[8];
            const f32x4 v0 = *reinterpret_cast<const f32x4 *>(&patch[r * PS + c]);
            const f32x4 v1 = *reinterpret_cast<const f32x4 *>(&patch[r * PS + c + 4]);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
              v[t] = v0[t];
              v[4 + t] = v1[t];
            }
            if (mt + 16 * hf + r < a.M && ntc + c < a.N) epilogue_store8(a, mt + 16 * hf + r, ntc + c, v, store_epi);
            __builtin_amdgcn_wave_barrier();
          }
        } else {
#pragma unroll
          for (int t = 0; t < 16; ++t) {
            const int m = mt + 8 * (t >> 2) + 4 * (lane >> 5) + (t & 3);
            const int n = ntc + (lane & 31);
            if (m < a.M && n < a.N)
              epilogue_store(a, m, n, acc[t]);
            else if (m < a.M && n < a.out_pad)
              store_f32(a.out, a.out_dtype, (size_t)m * a.out_ld + n, 0.f);
          }
        }
      }
    __syncthreads();  // every wave is done reading this A tile
    if (next < n_tiles) sstore(buf ^ 1);
    __syncthreads();
  }
}

template <int WN, int KS, bool GCNF>
static int launch_ws_k(const GemmNtArgs &a, hipStream_t s) {
  constexpr int TM = 64 * (4 / WN), LDK = KS * 16 + 8;
  const size_t smem = (size_t)2 * TM * LDK * sizeof(bf16_t) + (size_t)4 * 16 * 40 * sizeof(float);
  static bool attr_done = false;
  if (!attr_done) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_nt_bf16_ws_kernel<WN, KS, GCNF>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    attr_done = true;
  }
  const int n_tiles = (a.M + TM - 1) / TM;
  const int blocks = n_tiles < 512 ? n_tiles : 512;  // two persistent workgroups per compute unit
  hipLaunchKernelGGL((gemm_nt_bf16_ws_kernel<WN, KS, GCNF>), dim3(blocks), dim3(256), smem, s, a);
  return (int)hipGetLastError();
}

template <int WN, int KS>
static int launch_ws(const GemmNtArgs &a, hipStream_t s) {
  if (a.epilogue == EPI_FWD_GCN && a.vec_epi) return launch_ws_k<WN, KS, true>(a, s);
  return launch_ws_k<WN, KS, false>(a, s);
}

// ------------------------------------------------------------------------------------ bf16 TN
constexpr int TR = 64;      // reduction rows per step (two 16 KB operand tiles in flight per workgroup)
constexpr int LDS_P = 132;  // padded stride, in words, of one row pair of an LDS tile

// Both operands of the TN product are read along the reduction index (rows of A and of B), which is the slow
// index of their row-major tiles.  The LDS tiles therefore hold ROW PAIRS: word [p][c] is (row 2p, row 2p+1) of
// column c, so that the eight reduction elements of a matrix-core fragment are four 32-bit reads down one column.
__device__ __forceinline__ void store_row_pair(uint32_t *dst, const bf16x8 &even, const bf16x8 &odd) {
  const u32x4 x = __builtin_bit_cast(u32x4, even), y = __builtin_bit_cast(u32x4, odd);
  u32x4 lo, hi;
#pragma unroll
  for (int w = 0; w < 2; ++w) {
    lo[2 * w] = __builtin_amdgcn_perm(y[w], x[w], 0x05040100u);
    lo[2 * w + 1] = __builtin_amdgcn_perm(y[w], x[w], 0x07060302u);
    hi[2 * w] = __builtin_amdgcn_perm(y[w + 2], x[w + 2], 0x05040100u);
    hi[2 * w + 1] = __builtin_amdgcn_perm(y[w + 2], x[w + 2], 0x07060302u);
  }
  *reinterpret_cast<u32x4 *>(dst) = lo;
  *reinterpret_cast<u32x4 *>(dst + 4) = hi;
}

// PAIR: fp32 A with an even leading dimension and an 8-byte aligned base; a tile row (128 floats) is read by
// one wave instruction as 64 float pairs.
template <typename TA, bool VEC, bool PAIR = false>
__global__ __launch_bounds__(256) void gemm_tn_bf16_kernel(const GemmTnArgs a, int rows_per_split, int splits) {
  __shared__ __attribute__((aligned(16))) uint32_t As[TR / 2 * LDS_P];
  __shared__ __attribute__((aligned(16))) uint32_t Bs[TR / 2 * LDS_P];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  // XCD-aware order: the output tiles that read the same rows of A and B sit on one XCD (one L2)
  const int ti = (a.I + 127) / 128, tiles = ti * ((a.O + 127) / 128);
  const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
  const int tile = q % tiles, split = (q / tiles) * 8 + xcd;
  if (split >= splits) return;
  const int i0 = (tile % ti) * 128, o0 = (tile / ti) * 128;
  const int wi = (wave >> 1) * 64, wo = (wave & 1) * 64;
  const int r_begin = split * rows_per_split;
  const int r_end = min(a.M, r_begin + rows_per_split);
  const TA *A = static_cast<const TA *>(a.A);
  const bf16_t *B = static_cast<const bf16_t *>(a.B);
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  const int a_cols = VEC ? a.lda : a.I;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int t = 0; t < 16; ++t) acc[i][j][t] = 0.f;

  // bias gradient on the side: a product with an all-ones A fragment leaves the column sums of the B
  // tile in every row of its result; done by the waves that own the first rows of the first row tile
  const bool do_bias = a.bias_partial != nullptr && i0 == 0 && wi == 0;
  const bf16x8 ones8 = {(bf16_t)1.f, (bf16_t)1.f, (bf16_t)1.f, (bf16_t)1.f, (bf16_t)1.f, (bf16_t)1.f, (bf16_t)1.f, (bf16_t)1.f};
  f32x16 accb[2];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int t = 0; t < 16; ++t) accb[j][t] = 0.f;
  constexpr int NVT = TR * 16 / 256;  // 16-byte vectors per thread and operand tile
  bf16x8 ra[NVT], rb[NVT];
  constexpr int NPR = TR / 4;  // rows per wave and tile in the pair layout
  f32x2 rp[PAIR ? NPR : 1];
  auto gload = [&](int r0) {
    if constexpr (PAIR) {
#pragma unroll
      for (int i = 0; i < NPR; ++i) {
        const int r = 2 * (wave + 4 * (i >> 1)) + (i & 1), c = i0 + 2 * lane;
        f32x2 v = {0.f, 0.f};
        if (r0 + r < r_end) {
          const float *p = reinterpret_cast<const float *>(A) + (size_t)(r0 + r) * a.lda + c;
          if (c + 1 < a.I)
            v = *reinterpret_cast<const f32x2 *>(p);
          else if (c < a.I)
            v[0] = p[0];
        }
        rp[i] = v;
      }
    }
#pragma unroll
    for (int i = 0; i < NVT; ++i) {
      const int r = 2 * ((tid >> 4) + 16 * (i >> 1)) + (i & 1), c = (tid & 15) * 8;  // slots 2h, 2h+1: one row pair
      const bool rv = r0 + r < r_end;
      if constexpr (!PAIR) ra[i] = rv ? load8_bf16<TA, VEC>(A, (size_t)a.lda, r0 + r, i0 + c, a_cols) : zero8;
      rb[i] = (rv && o0 + c < a.ldb) ? *reinterpret_cast<const bf16x8 *>(B + (size_t)(r0 + r) * a.ldb + o0 + c) : zero8;
    }
  };
  if (r_begin < r_end) gload(r_begin);
  for (int r0 = r_begin; r0 < r_end; r0 += TR) {
    __syncthreads();  // previous step's fragment reads are done
    if constexpr (PAIR) {
#pragma unroll
      for (int h = 0; h < NPR / 2; ++h) {
        const bf16x2 c0 = {(bf16_t)rp[2 * h][0], (bf16_t)rp[2 * h + 1][0]};
        const bf16x2 c1 = {(bf16_t)rp[2 * h][1], (bf16_t)rp[2 * h + 1][1]};
        const u32x2 v = {__builtin_bit_cast(uint32_t, c0), __builtin_bit_cast(uint32_t, c1)};
        *reinterpret_cast<u32x2 *>(&As[(wave + 4 * h) * LDS_P + 2 * lane]) = v;
      }
    }
#pragma unroll
    for (int h = 0; h < NVT / 2; ++h) {
      const int p = (tid >> 4) + 16 * h, c = (tid & 15) * 8;
      if constexpr (!PAIR) store_row_pair(&As[p * LDS_P + c], ra[2 * h], ra[2 * h + 1]);
      store_row_pair(&Bs[p * LDS_P + c], rb[2 * h], rb[2 * h + 1]);
    }
    __syncthreads();
    if (r0 + TR < r_end) gload(r0 + TR);  // next tile's loads fly while this one is multiplied
#pragma unroll
    for (int kk = 0; kk < TR / 16; ++kk) {
      const int poff = kk * 8 + (lane >> 5) * 4;  // first of the fragment's four row pairs
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        u32x4 w;
#pragma unroll
        for (int t = 0; t < 4; ++t) w[t] = As[(poff + t) * LDS_P + wi + i * 32 + (lane & 31)];
        fa[i] = __builtin_bit_cast(bf16x8, w);
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        u32x4 w;
#pragma unroll
        for (int t = 0; t < 4; ++t) w[t] = Bs[(poff + t) * LDS_P + wo + j * 32 + (lane & 31)];
        fb[j] = __builtin_bit_cast(bf16x8, w);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
      if (do_bias) {  // wave-uniform
#pragma unroll
        for (int j = 0; j < 2; ++j) accb[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones8, fb[j], accb[j], 0, 0, 0);
      }
    }
  }
  if (do_bias && lane < 32) {  // element 0 of lanes 0..31 is row 0 of the result: the column sums
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int oo = o0 + wo + j * 32 + lane;
      if (oo < a.O) a.bias_partial[(size_t)split * a.O + oo] = accb[j][0];
    }
  }
  float *P = a.partial + (size_t)split * a.I * a.O;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int t = 0; t < 16; ++t) {
        const int ii = i0 + wi + i * 32 + 8 * (t >> 2) + 4 * (lane >> 5) + (t & 3);
        const int oo = o0 + wo + j * 32 + (lane & 31);
        if (ii < a.I && oo < a.O) P[(size_t)ii * a.O + oo] = acc[i][j][t];
      }
}

// The same product for long operands of up to 256 x 256 outputs (one weight-gradient product per layer over all rows
// of a pass): ONE workgroup of eight waves owns a row split and the whole I x O output, so every operand row is read
// from memory once.  With 128 x 128 tiles the four tiles of a split each stream half of both operands and share them
// only in part through their XCD's L2 (measured on 10 M rows: 16.1 GB fetched for 10.2 GB of operands).  A wave owns
// 64 rows x 128 columns of the output (eight 32 x 32 accumulators); both operands are bf16 with 16-byte aligned rows.
constexpr int LDS_PW = 260;  // padded stride, in words, of one row pair of a 256-column LDS tile
__global__ __launch_bounds__(512) void gemm_tn_bf16_wide_kernel(const GemmTnArgs a, int rows_per_split, int splits) {
  __shared__ __attribute__((aligned(16))) uint32_t As[TR / 2 * LDS_PW];
  __shared__ __attribute__((aligned(16))) uint32_t Bs[TR / 2 * LDS_PW];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int split = blockIdx.x;
  if (split >= splits) return;
  const int wi = (wave >> 1) * 64, wo = (wave & 1) * 128;
  const int r_begin = split * rows_per_split;
  const int r_end = min(a.M, r_begin + rows_per_split);
  const bf16_t *A = static_cast<const bf16_t *>(a.A);
  const bf16_t *B = static_cast<const bf16_t *>(a.B);
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};

  f32x16 acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int t = 0; t < 16; ++t) acc[i][j][t] = 0.f;
  // bias gradient on the side: every thread adds up the B rows it stages (its 8 columns, 4 rows per tile); the 16
  // threads that share a column group are added in a fixed order at the end.  (The all-ones matrix product of the
  // 128 x 128 kernel would cost 64 more accumulator registers here.)
  const bool do_bias = a.bias_partial != nullptr;
  float bsum[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) bsum[t] = 0.f;
  constexpr int NVT = TR * 32 / 512;  // 16-byte vectors per thread and operand tile
  bf16x8 ra[NVT], rb[NVT];
  const int c = (tid & 31) * 8;
  auto gload = [&](int r0) {
#pragma unroll
    for (int i = 0; i < NVT; ++i) {
      const int r = 2 * ((tid >> 5) + 16 * (i >> 1)) + (i & 1);  // slots 2h, 2h+1: one row pair
      const bool rv = r0 + r < r_end;
      ra[i] = (rv && c < a.lda) ? *reinterpret_cast<const bf16x8 *>(A + (size_t)(r0 + r) * a.lda + c) : zero8;
      rb[i] = (rv && c < a.ldb) ? *reinterpret_cast<const bf16x8 *>(B + (size_t)(r0 + r) * a.ldb + c) : zero8;
    }
  };
  if (r_begin < r_end) gload(r_begin);
  for (int r0 = r_begin; r0 < r_end; r0 += TR) {
    __syncthreads();  // previous step's fragment reads are done
#pragma unroll
    for (int h = 0; h < NVT / 2; ++h) {
      const int p = (tid >> 5) + 16 * h;
      store_row_pair(&As[p * LDS_PW + c], ra[2 * h], ra[2 * h + 1]);
      store_row_pair(&Bs[p * LDS_PW + c], rb[2 * h], rb[2 * h + 1]);
    }
    if (do_bias) {
#pragma unroll
      for (int i = 0; i < NVT; ++i)
#pragma unroll
        for (int t = 0; t < 8; ++t) bsum[t] += (float)rb[i][t];
    }
    __syncthreads();
    if (r0 + TR < r_end) gload(r0 + TR);  // next tile's loads fly while this one is multiplied
#pragma unroll
    for (int kk = 0; kk < TR / 16; ++kk) {
      const int poff = kk * 8 + (lane >> 5) * 4;  // first of the fragment's four row pairs
      bf16x8 fa[2], fb[4];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        u32x4 w;
#pragma unroll
        for (int t = 0; t < 4; ++t) w[t] = As[(poff + t) * LDS_PW + wi + i * 32 + (lane & 31)];
        fa[i] = __builtin_bit_cast(bf16x8, w);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        u32x4 w;
#pragma unroll
        for (int t = 0; t < 4; ++t) w[t] = Bs[(poff + t) * LDS_PW + wo + j * 32 + (lane & 31)];
        fb[j] = __builtin_bit_cast(bf16x8, w);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  }
  if (do_bias) {
    __syncthreads();  // the operand tiles are done with; As is reused for the threads' column sums
    float *cs = reinterpret_cast<float *>(As);
    static_assert(512 * 8 * sizeof(float) <= sizeof(As), "the column sums must fit the A tile");
#pragma unroll
    for (int t = 0; t < 8; ++t) cs[tid * 8 + t] = bsum[t];
    __syncthreads();
    if (tid < 256 && tid < a.O) {  // column tid: the threads (g * 32 + tid / 8), g = 0 .. 15, element tid % 8
      float sum = 0.f;
#pragma unroll
      for (int g = 0; g < 16; ++g) sum += cs[(g * 32 + (tid >> 3)) * 8 + (tid & 7)];
      a.bias_partial[(size_t)split * a.O + tid] = sum;
    }
  }
  float *P = a.partial + (size_t)split * a.I * a.O;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int t = 0; t < 16; ++t) {
        const int ii = wi + i * 32 + 8 * (t >> 2) + 4 * (lane >> 5) + (t & 3);
        const int oo = wo + j * 32 + (lane & 31);
        if (ii < a.I && oo < a.O) P[(size_t)ii * a.O + oo] = acc[i][j][t];
      }
}

// ------------------------------------------------------------------------------------ fp32 NT
template <bool VEC>
__global__ __launch_bounds__(256) void gemm_nt_f32_kernel(const GemmNtArgs a) {
  constexpr int T = 64, KB = 16;
  __shared__ float As[KB][T + 4];
  __shared__ float Bs[KB][T + 4];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.x * T, n0 = blockIdx.y * T;
  const float *A = static_cast<const float *>(a.A);
  const float *Bt = static_cast<const float *>(a.Bt);
  float acc[4][4] = {};
  const int lr = tid >> 2, lk = (tid & 3) * 4;
  for (int k0 = 0; k0 < a.Kp; k0 += KB) {
    f32x4 va = {0.f, 0.f, 0.f, 0.f}, vb = {0.f, 0.f, 0.f, 0.f};
    if (m0 + lr < a.M) {
      const float *p = A + (size_t)(m0 + lr) * a.lda + k0 + lk;
      if constexpr (VEC) {
        if (k0 + lk < a.Kp) va = *reinterpret_cast<const f32x4 *>(p);
      } else {
#pragma unroll
        for (int t = 0; t < 4; ++t)
          if (k0 + lk + t < a.K) va[t] = p[t];
      }
    }
    if (n0 + lr < a.N && k0 + lk < a.Kp) vb = *reinterpret_cast<const f32x4 *>(Bt + (size_t)(n0 + lr) * a.ldb + k0 + lk);
    __syncthreads();
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      As[lk + t][lr] = va[t];
      Bs[lk + t][lr] = vb[t];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < KB; ++k) {
      float x[4], y[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        x[t] = As[k][ty * 4 + t];
        y[t] = Bs[k][tx * 4 + t];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += x[i] * y[j];
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < a.M && n < a.N)
        epilogue_store(a, m, n, acc[i][j]);
      else if (m < a.M && n < a.out_pad)
        store_f32(a.out, a.out_dtype, (size_t)m * a.out_ld + n, 0.f);
    }
}

// ------------------------------------------------------------------------------------ fp32 TN
template <bool VEC>
__global__ __launch_bounds__(256) void gemm_tn_f32_kernel(const GemmTnArgs a, int rows_per_split) {
  constexpr int T = 64, RB = 16;
  __shared__ float As[RB][T + 4];
  __shared__ float Bs[RB][T + 4];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int i0 = blockIdx.x * T, o0 = blockIdx.y * T;
  const int r_begin = blockIdx.z * rows_per_split;
  const int r_end = min(a.M, r_begin + rows_per_split);
  const float *A = static_cast<const float *>(a.A);
  const float *B = static_cast<const float *>(a.B);
  float acc[4][4] = {};
  const int lr = tid >> 4, lc = (tid & 15) * 4;
  for (int r0 = r_begin; r0 < r_end; r0 += RB) {
    f32x4 va = {0.f, 0.f, 0.f, 0.f}, vb = {0.f, 0.f, 0.f, 0.f};
    if (r0 + lr < r_end) {
      const float *p = A + (size_t)(r0 + lr) * a.lda + i0 + lc;
      if constexpr (VEC) {
        if (i0 + lc < a.lda) va = *reinterpret_cast<const f32x4 *>(p);
      } else {
#pragma unroll
        for (int t = 0; t < 4; ++t)
          if (i0 + lc + t < a.I) va[t] = p[t];
      }
      if (o0 + lc < a.ldb) vb = *reinterpret_cast<const f32x4 *>(B + (size_t)(r0 + lr) * a.ldb + o0 + lc);
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      As[lr][lc + t] = va[t];
      Bs[lr][lc + t] = vb[t];
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      float x[4], y[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        x[t] = As[r][ty * 4 + t];
        y[t] = Bs[r][tx * 4 + t];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += x[i] * y[j];
    }
  }
  float *P = a.partial + (size_t)blockIdx.z * a.I * a.O;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int ii = i0 + ty * 4 + i, oo = o0 + tx * 4 + j;
      if (ii < a.I && oo < a.O) P[(size_t)ii * a.O + oo] = acc[i][j];
    }
}

// dst[e] += scale * sum_s partial[s][e].  Fixed summation order => reproducible.  64 outputs per block,
// four phases of splits summed in parallel (8 independent loads in flight each), then combined in LDS.
// A second sum over the same splits (the bias gradient next to a weight gradient) rides in the same launch:
// blocks from blocks1 on serve (partial2, count2, dst2) with scale 1.
__global__ __launch_bounds__(256) void reduce_add_kernel(const float *partial, int splits, size_t count, float scale,
                                                         float *dst, unsigned blocks1, const float *partial2, size_t count2,
                                                         float *dst2) {
  __shared__ float red[4][64];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  unsigned block = blockIdx.x;
  if (block >= blocks1) {  // whole workgroup
    block -= blocks1;
    partial = partial2;
    count = count2;
    scale = 1.0f;
    dst = dst2;
  }
  const size_t e = (size_t)block * 64 + tx;
  float s = 0.f;
  if (e < count) {
    const int per = (splits + 3) / 4;
    const int k0 = ty * per, k1 = min(splits, k0 + per);
    int k = k0;
    for (; k + 8 <= k1; k += 8) {
      float v[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) v[t] = partial[(size_t)(k + t) * count + e];
#pragma unroll
      for (int t = 0; t < 8; ++t) s += v[t];
    }
    for (; k < k1; ++k) s += partial[(size_t)k * count + e];
  }
  red[ty][tx] = s;
  __syncthreads();
  if (ty == 0 && e < count) dst[e] += scale * ((red[0][tx] + red[1][tx]) + (red[2][tx] + red[3][tx]));
}

// partial[split][o] = sum of B[r][o] over the split's rows: 64 columns x 4 row phases per block
template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(const T *B, int ldb, int M, int O, int rows_per_split, float *partial) {
  __shared__ float red[4][64];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int o = blockIdx.x * 64 + tx;
  const int r_begin = blockIdx.y * rows_per_split;
  const int r_end = min(M, r_begin + rows_per_split);
  float s = 0.f;
  if (o < O)
    for (int r = r_begin + ty; r < r_end; r += 4) s += to_f32(B[(size_t)r * ldb + o]);
  red[ty][tx] = s;
  __syncthreads();
  if (ty == 0 && o < O) partial[(size_t)blockIdx.y * O + o] = (red[0][tx] + red[1][tx]) + (red[2][tx] + red[3][tx]);
}

// Same sums with 16-byte loads of 8 bf16 columns: 32 column vectors x 8 row phases per block, two rows
// in flight per thread.  Needs ldb % 8 == 0 and a 16-byte aligned base (the library's padded buffers).
__global__ __launch_bounds__(256) void colsum_bf16_vec_kernel(const bf16_t *B, int ldb, int M, int O, int rows_per_split,
                                                              float *partial) {
  __shared__ float red[8][32][8];
  const int cv = threadIdx.x & 31, ph = threadIdx.x >> 5;
  const int o = (blockIdx.x * 32 + cv) * 8;
  const int r_begin = blockIdx.y * rows_per_split;
  const int r_end = min(M, r_begin + rows_per_split);
  float s[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) s[t] = 0.f;
  if (o < ldb) {
    int r = r_begin + ph;
    for (; r + 8 < r_end; r += 16) {
      const bf16x8 x0 = *reinterpret_cast<const bf16x8 *>(B + (size_t)r * ldb + o);
      const bf16x8 x1 = *reinterpret_cast<const bf16x8 *>(B + (size_t)(r + 8) * ldb + o);
#pragma unroll
      for (int t = 0; t < 8; ++t) s[t] += (float)x0[t];
#pragma unroll
      for (int t = 0; t < 8; ++t) s[t] += (float)x1[t];
    }
    for (; r < r_end; r += 8) {
      const bf16x8 x0 = *reinterpret_cast<const bf16x8 *>(B + (size_t)r * ldb + o);
#pragma unroll
      for (int t = 0; t < 8; ++t) s[t] += (float)x0[t];
    }
  }
#pragma unroll
  for (int t = 0; t < 8; ++t) red[ph][cv][t] = s[t];
  __syncthreads();
  if (ph == 0 && o < ldb) {
#pragma unroll
    for (int p = 1; p < 8; ++p)
#pragma unroll
      for (int t = 0; t < 8; ++t) s[t] += red[p][cv][t];
#pragma unroll
    for (int t = 0; t < 8; ++t)
      if (o + t < O) partial[(size_t)blockIdx.y * O + o + t] = s[t];
  }
}

bool vec_ok(const void *p, int ld, int mult) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0 && ld % mult == 0; }

}  // namespace

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static bool pair_ok(const void *p, int ld) { return (reinterpret_cast<uintptr_t>(p) & 7u) == 0 && ld % 2 == 0; }

int launch_gemm_nt(const GemmNtArgs &a_in, int compute_dtype, hipStream_t s) {
  if (a_in.M <= 0 || a_in.N <= 0) return hipSuccess;
  GemmNtArgs a = a_in;
  const bool has_aux = a.epilogue == EPI_FWD_GCNII || a.epilogue == EPI_MASK || a.epilogue == EPI_DGRAD_GCNII ||
                       a.epilogue == EPI_FWD_ADD || a.epilogue == EPI_RES;
  a.vec_epi = a.N % 8 == 0 && a.out_ld % 8 == 0 && aligned16(a.out) && (a.out_pad <= a.N) &&
              (!has_aux || (a.aux_ld % 8 == 0 && aligned16(a.aux))) &&
              ((a.epilogue != EPI_FWD_GCN && a.epilogue != EPI_FWD_ADD && a.epilogue != EPI_RES) || aligned16(a.bias)) &&
              (a.epilogue != EPI_DGRAD_GCNII || !a.h0grad || (a.h0_ld % 4 == 0 && aligned16(a.h0grad)));
  if (compute_dtype == DT_BF16) {
    const int mt = (a.M + BM - 1) / BM, ntiles = (a.N + BN - 1) / BN;
    dim3 grid((unsigned)(((mt + 7) / 8) * 8 * ntiles));
    const bool vec = a.a_dtype == DT_BF16 && vec_ok(a.A, a.lda, 8) && a.lda >= a.Kp;
    if (a.a_dtype == DT_F32 && pair_ok(a.A, a.lda))
      hipLaunchKernelGGL((gemm_nt_bf16_kernel<float, false, true>), grid, dim3(256), 0, s, a);
    else if (a.a_dtype == DT_F32)
      hipLaunchKernelGGL((gemm_nt_bf16_kernel<float, false>), grid, dim3(256), 0, s, a);
    else if (vec && vec_ok(a.Bt, a.ldb, 8) && a.Kp <= 256 && a.N <= 256 && a.M >= a.ws_min_rows) {
      // long operands: persistent weight-stationary kernel (needs a few row tiles per workgroup to pay
      // for loading its panel of Bt into registers)
      if (a.N <= 128 && a.Kp <= 128) return launch_ws<2, 8>(a, s);
      if (a.N <= 128) return launch_ws<2, 16>(a, s);
      if (a.Kp <= 128) return launch_ws<4, 8>(a, s);
      return launch_ws<4, 16>(a, s);
    } else if (vec && a.Kp >= 128 && (long long)mt * ntiles <= 1024)
      // short operands: every workgroup is resident at once, the product is its chain of K steps
      hipLaunchKernelGGL((gemm_nt_bf16_kernel<bf16_t, true, false, 64>), grid, dim3(256), 0, s, a);
    else if (vec)
      hipLaunchKernelGGL((gemm_nt_bf16_kernel<bf16_t, true>), grid, dim3(256), 0, s, a);
    else
      hipLaunchKernelGGL((gemm_nt_bf16_kernel<bf16_t, false>), grid, dim3(256), 0, s, a);
  } else {
    if (a.a_dtype != DT_F32) return hipErrorInvalidValue;
    dim3 grid((a.M + 63) / 64, (a.N + 63) / 64);
    if (vec_ok(a.A, a.lda, 4) && a.lda >= a.Kp)
      hipLaunchKernelGGL(gemm_nt_f32_kernel<true>, grid, dim3(256), 0, s, a);
    else
      hipLaunchKernelGGL(gemm_nt_f32_kernel<false>, grid, dim3(256), 0, s, a);
  }
  return (int)hipGetLastError();
}

int launch_gemm_tn(const GemmTnArgs &a, int compute_dtype, hipStream_t s) {
  if (a.M <= 0 || a.I <= 0 || a.O <= 0) return hipSuccess;
  const int tile = compute_dtype == DT_BF16 ? 128 : 64;
  const int step = compute_dtype == DT_BF16 ? TR : 16;
  const int ti = (a.I + tile - 1) / tile, to = (a.O + tile - 1) / tile;
  int splits = 1024 / (ti * to);  // about four blocks per compute unit ...
  // ... but the fp32 partials (write + read, 8 bytes per output element and split) should not move more than
  // twice the operands themselves (2 bytes per element of A and B); below that the kernel is latency-bound and
  // more blocks win
  const long long cap = (long long)a.M * (a.I + a.O) / (2LL * a.I * a.O);
  if (splits > cap) splits = (int)cap;
  if (splits < 1) splits = 1;
  if (splits > a.max_splits) splits = a.max_splits;
  int rows_per = (a.M + splits - 1) / splits;
  rows_per = (rows_per + step - 1) / step * step;
  splits = (a.M + rows_per - 1) / rows_per;
  dim3 grid(ti, to, splits);
  // long operands with more than one 128 x 128 output tile: one workgroup per row split computes all of the output
  const bool wide = compute_dtype == DT_BF16 && a.a_dtype == DT_BF16 && a.M >= a.wide_min_rows && ti * to > 1 && a.I <= 256 &&
                    a.O <= 256 && vec_ok(a.A, a.lda, 8) && vec_ok(a.B, a.ldb, 8);
  if (wide) {
    splits = a.max_splits < 256 ? a.max_splits : 256;  // one workgroup per compute unit
    rows_per = (a.M + splits - 1) / splits;
    rows_per = (rows_per + step - 1) / step * step;
    splits = (a.M + rows_per - 1) / rows_per;
    hipLaunchKernelGGL(gemm_tn_bf16_wide_kernel, dim3((unsigned)splits), dim3(512), 0, s, a, rows_per, splits);
  } else if (compute_dtype == DT_BF16) {
    dim3 g1((unsigned)(((splits + 7) / 8) * 8 * ti * to));
    if (a.a_dtype == DT_F32 && pair_ok(a.A, a.lda))
      hipLaunchKernelGGL((gemm_tn_bf16_kernel<float, false, true>), g1, dim3(256), 0, s, a, rows_per, splits);
    else if (a.a_dtype == DT_F32)
      hipLaunchKernelGGL((gemm_tn_bf16_kernel<float, false>), g1, dim3(256), 0, s, a, rows_per, splits);
    else if (vec_ok(a.A, a.lda, 8))
      hipLaunchKernelGGL((gemm_tn_bf16_kernel<bf16_t, true>), g1, dim3(256), 0, s, a, rows_per, splits);
    else
      hipLaunchKernelGGL((gemm_tn_bf16_kernel<bf16_t, false>), g1, dim3(256), 0, s, a, rows_per, splits);
  } else {
    if (a.a_dtype != DT_F32) return hipErrorInvalidValue;
    if (vec_ok(a.A, a.lda, 4))
      hipLaunchKernelGGL(gemm_tn_f32_kernel<true>, grid, dim3(256), 0, s, a, rows_per);
    else
      hipLaunchKernelGGL(gemm_tn_f32_kernel<false>, grid, dim3(256), 0, s, a, rows_per);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return (int)e;
  const size_t count = (size_t)a.I * a.O;
  if (a.dbias != nullptr && compute_dtype != DT_BF16) return hipErrorInvalidValue;  // the fp32 stage sums columns separately
  const unsigned blocks1 = (unsigned)((count + 63) / 64), blocks2 = a.dbias != nullptr ? (unsigned)((a.O + 63) / 64) : 0u;
  hipLaunchKernelGGL(reduce_add_kernel, dim3(blocks1 + blocks2), dim3(256), 0, s, a.partial, splits, count, a.scale, a.dW, blocks1,
                     a.bias_partial, (size_t)a.O, a.dbias);
  return (int)hipGetLastError();
}

int launch_colsum_add(const void *B, int dtype, int ldb, int M, int O, float *partial, int max_splits, float *dst,
                      hipStream_t s) {
  if (M <= 0 || O <= 0) return hipSuccess;
  int splits = (M + 255) / 256;
  if (splits > max_splits) splits = max_splits;
  const int rows_per = (M + splits - 1) / splits;
  splits = (M + rows_per - 1) / rows_per;
  dim3 grid((O + 63) / 64, splits);
  if (dtype == DT_BF16 && vec_ok(B, ldb, 8))
    hipLaunchKernelGGL(colsum_bf16_vec_kernel, dim3((ldb / 8 + 31) / 32, splits), dim3(256), 0, s,
                       static_cast<const bf16_t *>(B), ldb, M, O, rows_per, partial);
  else if (dtype == DT_BF16)
    hipLaunchKernelGGL(colsum_kernel<bf16_t>, grid, dim3(256), 0, s, static_cast<const bf16_t *>(B), ldb, M, O, rows_per, partial);
  else
    hipLaunchKernelGGL(colsum_kernel<float>, grid, dim3(256), 0, s, static_cast<const float *>(B), ldb, M, O, rows_per, partial);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return (int)e;
  hipLaunchKernelGGL(reduce_add_kernel, dim3((unsigned)((O + 63) / 64)), dim3(256), 0, s, partial, splits, (size_t)O, 1.0f, dst,
                     (unsigned)((O + 63) / 64), static_cast<const float *>(nullptr), (size_t)0, static_cast<float *>(nullptr));
  return (int)hipGetLastError();
}
