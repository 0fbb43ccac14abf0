// Dense transforms of the stage (the UPDATE line of Algorithm 1 and its gradients).
//
//   NT:  C[M x N]  = A[M x Kp] . Bt[N x Kp]^T     forward transform and input gradient
//   TN:  dW[I x O] += s * A[M x I]^T . B[M x O]    weight gradient (reduction over chunk rows)
//
// bf16 operands go through the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32
// accumulation); the fp32 variants are plain LDS-tiled FMA kernels used by the fp32 stage.
// Bias / ReLU / GCNII residual terms are applied in the epilogue on the fp32 accumulators.
#include "common.h"

namespace {

typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ inline float to_f32(float x) { return x; }
__device__ inline float to_f32(bf16_t x) { return (float)x; }
template <typename T>
__device__ inline T from_f32(float x);
template <>
__device__ inline float from_f32<float>(float x) { return x; }
template <>
__device__ inline bf16_t from_f32<bf16_t>(float x) { return (bf16_t)x; }

// One output element of an NT product: epilogue + store.  T is both the dtype of aux and of out.
template <typename T>
__device__ inline void epilogue_store(const GemmNtArgs &a, int m, int n, float acc) {
  float r;
  switch (a.epilogue) {
    case EPI_FWD_GCN: {
      r = acc + a.bias[n];
      r = r > 0.f ? r : 0.f;
      break;
    }
    case EPI_FWD_GCNII: {
      const float p = to_f32(static_cast<const T *>(a.aux)[(size_t)m * a.aux_ld + n]);
      r = (1.f - a.beta) * p + a.beta * acc;
      r = r > 0.f ? r : 0.f;
      break;
    }
    case EPI_DGRAD_GCN: {
      r = acc;
      break;
    }
    default: {  // EPI_DGRAD_GCNII
      const float dy = to_f32(static_cast<const T *>(a.aux)[(size_t)m * a.aux_ld + n]);
      const float dp = (1.f - a.beta) * dy + a.beta * acc;
      r = (1.f - a.alpha) * dp;
      if (a.h0grad) a.h0grad[(size_t)m * a.h0_ld + n] += a.alpha * dp;
      break;
    }
  }
  static_cast<T *>(a.out)[(size_t)m * a.out_ld + n] = from_f32<T>(r);
}

// ------------------------------------------------------------------------------------ bf16 NT
constexpr int BM = 128, BN = 128, BK = 32;
constexpr int LDS_K = 40;  // padded K stride (elements): 80-byte rows keep 16-byte fragment reads conflict-free

__global__ __launch_bounds__(256) void gemm_nt_bf16_kernel(const GemmNtArgs a) {
  __shared__ __attribute__((aligned(16))) bf16_t As[2][BM * LDS_K];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[2][BN * LDS_K];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
  const bf16_t *A = static_cast<const bf16_t *>(a.A);
  const bf16_t *Bt = static_cast<const bf16_t *>(a.Bt);

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int t = 0; t < 16; ++t) acc[i][j][t] = 0.f;

  bf16x8 ra[2], rb[2];
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  auto gload = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int vid = tid + 256 * i, r = vid >> 2, k = k0 + (vid & 3) * 8;
      ra[i] = (m0 + r < a.M && k < a.Kp) ? *reinterpret_cast<const bf16x8 *>(A + (size_t)(m0 + r) * a.lda + k) : zero8;
      rb[i] = (n0 + r < a.N && k < a.Kp) ? *reinterpret_cast<const bf16x8 *>(Bt + (size_t)(n0 + r) * a.ldb + k) : zero8;
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int vid = tid + 256 * i, r = vid >> 2, kv = vid & 3;
      *reinterpret_cast<bf16x8 *>(&As[buf][r * LDS_K + kv * 8]) = ra[i];
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
  // 32x32 accumulator layout: element t of lane l is row 8*(t/4) + 4*(l/32) + t%4, column l%32
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int t = 0; t < 16; ++t) {
        const int m = m0 + wm + i * 32 + 8 * (t >> 2) + 4 * (lane >> 5) + (t & 3);
        const int n = n0 + wn + j * 32 + (lane & 31);
        if (m < a.M && n < a.N) epilogue_store<bf16_t>(a, m, n, acc[i][j][t]);
      }
}

// ------------------------------------------------------------------------------------ bf16 TN
constexpr int TR = 32;      // reduction rows per step
constexpr int LDS_C = 136;  // padded column stride of the row-major LDS tiles

__global__ __launch_bounds__(256) void gemm_tn_bf16_kernel(const GemmTnArgs a, int rows_per_split) {
  __shared__ __attribute__((aligned(16))) bf16_t As[TR * LDS_C];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[TR * LDS_C];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int i0 = blockIdx.x * 128, o0 = blockIdx.y * 128;
  const int wi = (wave >> 1) * 64, wo = (wave & 1) * 64;
  const int r_begin = blockIdx.z * rows_per_split;
  const int r_end = min(a.M, r_begin + rows_per_split);
  const bf16_t *A = static_cast<const bf16_t *>(a.A);
  const bf16_t *B = static_cast<const bf16_t *>(a.B);
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int t = 0; t < 16; ++t) acc[i][j][t] = 0.f;

  for (int r0 = r_begin; r0 < r_end; r0 += TR) {
    bf16x8 ra[2], rb[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int vid = tid + 256 * i, r = vid >> 4, c = (vid & 15) * 8;
      const bool rv = r0 + r < r_end;
      ra[i] = (rv && i0 + c < a.lda) ? *reinterpret_cast<const bf16x8 *>(A + (size_t)(r0 + r) * a.lda + i0 + c) : zero8;
      rb[i] = (rv && o0 + c < a.ldb) ? *reinterpret_cast<const bf16x8 *>(B + (size_t)(r0 + r) * a.ldb + o0 + c) : zero8;
    }
    __syncthreads();  // previous step's fragment reads are done
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int vid = tid + 256 * i, r = vid >> 4, c = (vid & 15) * 8;
      *reinterpret_cast<bf16x8 *>(&As[r * LDS_C + c]) = ra[i];
      *reinterpret_cast<bf16x8 *>(&Bs[r * LDS_C + c]) = rb[i];
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TR / 16; ++kk) {
      const int roff = kk * 16 + (lane >> 5) * 8;
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int t = 0; t < 8; ++t) fa[i][t] = As[(roff + t) * LDS_C + wi + i * 32 + (lane & 31)];
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int t = 0; t < 8; ++t) fb[j][t] = Bs[(roff + t) * LDS_C + wo + j * 32 + (lane & 31)];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  }
  float *P = a.partial + (size_t)blockIdx.z * a.I * a.O;
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

// ------------------------------------------------------------------------------------ fp32 NT
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
    if (m0 + lr < a.M && k0 + lk < a.Kp) va = *reinterpret_cast<const f32x4 *>(A + (size_t)(m0 + lr) * a.lda + k0 + lk);
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
      if (m < a.M && n < a.N) epilogue_store<float>(a, m, n, acc[i][j]);
    }
}

// ------------------------------------------------------------------------------------ fp32 TN
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
    if (r0 + lr < r_end && i0 + lc < a.lda) va = *reinterpret_cast<const f32x4 *>(A + (size_t)(r0 + lr) * a.lda + i0 + lc);
    if (r0 + lr < r_end && o0 + lc < a.ldb) vb = *reinterpret_cast<const f32x4 *>(B + (size_t)(r0 + lr) * a.ldb + o0 + lc);
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

// dst[e] += scale * sum_s partial[s][e]   (fixed summation order => reproducible)
__global__ __launch_bounds__(256) void reduce_add_kernel(const float *partial, int splits, size_t count, float scale,
                                                         float *dst) {
  const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= count) return;
  float s = 0.f;
  for (int k = 0; k < splits; ++k) s += partial[(size_t)k * count + e];
  dst[e] += scale * s;
}

// partial[split][o] = sum of B[r][o] over the split's rows
template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(const T *B, int ldb, int M, int O, int rows_per_split, float *partial) {
  const int o = blockIdx.x * 256 + threadIdx.x;
  if (o >= O) return;
  const int r_begin = blockIdx.y * rows_per_split;
  const int r_end = min(M, r_begin + rows_per_split);
  float s = 0.f;
  for (int r = r_begin; r < r_end; ++r) s += to_f32(B[(size_t)r * ldb + o]);
  partial[(size_t)blockIdx.y * O + o] = s;
}

}  // namespace

int launch_gemm_nt(const GemmNtArgs &a, int compute_dtype, int out_dtype, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0) return hipSuccess;
  if (compute_dtype != out_dtype) return hipErrorInvalidValue;
  if (compute_dtype == DT_BF16) {
    dim3 grid((a.M + BM - 1) / BM, (a.N + BN - 1) / BN);
    hipLaunchKernelGGL(gemm_nt_bf16_kernel, grid, dim3(256), 0, s, a);
  } else {
    dim3 grid((a.M + 63) / 64, (a.N + 63) / 64);
    hipLaunchKernelGGL(gemm_nt_f32_kernel, grid, dim3(256), 0, s, a);
  }
  return (int)hipGetLastError();
}

int launch_gemm_tn(const GemmTnArgs &a, int compute_dtype, hipStream_t s) {
  if (a.M <= 0 || a.I <= 0 || a.O <= 0) return hipSuccess;
  const int tile = compute_dtype == DT_BF16 ? 128 : 64;
  const int step = compute_dtype == DT_BF16 ? TR : 16;
  const int ti = (a.I + tile - 1) / tile, to = (a.O + tile - 1) / tile;
  int splits = 256 / (ti * to);
  if (splits < 1) splits = 1;
  if (splits > a.max_splits) splits = a.max_splits;
  int rows_per = (a.M + splits - 1) / splits;
  rows_per = (rows_per + step - 1) / step * step;
  splits = (a.M + rows_per - 1) / rows_per;
  dim3 grid(ti, to, splits);
  if (compute_dtype == DT_BF16)
    hipLaunchKernelGGL(gemm_tn_bf16_kernel, grid, dim3(256), 0, s, a, rows_per);
  else
    hipLaunchKernelGGL(gemm_tn_f32_kernel, grid, dim3(256), 0, s, a, rows_per);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return (int)e;
  const size_t count = (size_t)a.I * a.O;
  hipLaunchKernelGGL(reduce_add_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s, a.partial, splits, count,
                     a.scale, a.dW);
  e = hipGetLastError();
  if (e != hipSuccess) return (int)e;
  if (a.dbias != nullptr) {
    dim3 g2((a.O + 255) / 256, splits);
    if (compute_dtype == DT_BF16)
      hipLaunchKernelGGL(colsum_kernel<bf16_t>, g2, dim3(256), 0, s, static_cast<const bf16_t *>(a.B), a.ldb, a.M, a.O,
                         rows_per, a.bias_partial);
    else
      hipLaunchKernelGGL(colsum_kernel<float>, g2, dim3(256), 0, s, static_cast<const float *>(a.B), a.ldb, a.M, a.O,
                         rows_per, a.bias_partial);
    e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
    hipLaunchKernelGGL(reduce_add_kernel, dim3((unsigned)((a.O + 255) / 256)), dim3(256), 0, s, a.bias_partial, splits,
                       (size_t)a.O, 1.0f, a.dbias);
    e = hipGetLastError();
  }
  return (int)e;
}
