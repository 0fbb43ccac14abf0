// Row-wise LayerNorm + ReLU in front of the aggregation (ResGCN+ variant), its backward, and a row copy
// with padding.  One wavefront per vertex row; rows are strided over the launched wavefronts.
//
// LayerNorm over the d features of one vertex: y = gamma * (x - mean) / sqrt(var + eps) + beta with the
// biased variance; the layer's input to the aggregation is r = ReLU(y).
#include <hip/hip_runtime.h>

#include <algorithm>

#include "common.h"

namespace {

__device__ inline float ld_elt(const void *p, int dtype, size_t i) {
  return dtype == DT_BF16 ? (float)static_cast<const bf16_t *>(p)[i] : static_cast<const float *>(p)[i];
}
__device__ inline void st_elt(void *p, int dtype, size_t i, float v) {
  if (dtype == DT_BF16)
    static_cast<bf16_t *>(p)[i] = (bf16_t)v;
  else
    static_cast<float *>(p)[i] = v;
}

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// NI = columns per lane (lane, lane + 64, ...): the row lives in registers between the passes
template <int NI>
__global__ __launch_bounds__(256) void ln_relu_kernel(const void *x, int x_dtype, int x_ld, const float *gamma, const float *beta,
                                                      float eps, int64_t M, int d, void *out, int out_dtype, int out_ld,
                                                      const LnDropout dp) {
  const int lane = threadIdx.x & 63;
  const int64_t w0 = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), nw = (int64_t)gridDim.x * 4;
  for (int64_t r = w0; r < M; r += nw) {
    float v[NI];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int c = lane + 64 * i;
      v[i] = c < d ? ld_elt(x, x_dtype, (size_t)r * x_ld + c) : 0.f;
      sum += v[i];
    }
    const float mean = wave_sum(sum) / (float)d;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int c = lane + 64 * i;
      const float t = c < d ? v[i] - mean : 0.f;
      sq += t * t;
    }
    const float rstd = 1.f / sqrtf(wave_sum(sq) / (float)d + eps);
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int c = lane + 64 * i;
      if (c < out_ld) {
        float y = 0.f;
        if (c < d) {
          y = gamma[c] * ((v[i] - mean) * rstd) + beta[c];
          y = y > 0.f ? y : 0.f;
          if (dp.threshold > 0) y = dropout_keep(dp, dp.u0 + r, d, c) ? y * dp.scale : 0.f;
        }
        st_elt(out, out_dtype, (size_t)r * out_ld + c, y);
      }
    }
  }
}

// dr -> dx (+ res) for the rows of the launch; the column sums of the parameter gradients are added over the
// four wavefronts of a workgroup in LDS and go to partial[workgroup][0][c] (gamma) and partial[workgroup][1][c]
// (beta); ln_param_reduce_kernel adds those in a fixed order.
template <int NI>
__global__ __launch_bounds__(256) void ln_relu_backward_kernel(const void *x, int x_dtype, int x_ld, const float *gamma,
                                                               const float *beta, float eps, const void *dr, int dr_dtype, int dr_ld,
                                                               const void *res, int res_dtype, int res_ld, int64_t M, int d,
                                                               void *out, int out_dtype, int out_ld, float *partial,
                                                               const LnDropout dp) {
  __shared__ float red[3][2][NI * 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t w0 = (int64_t)blockIdx.x * 4 + wave, nw = (int64_t)gridDim.x * 4;
  float dg[NI], db[NI], gam[NI], bet[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int c = lane + 64 * i;
    dg[i] = db[i] = 0.f;
    gam[i] = c < d ? gamma[c] : 0.f;
    bet[i] = c < d ? beta[c] : 0.f;
  }
  for (int64_t r = w0; r < M; r += nw) {
    float xh[NI], dxh[NI];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int c = lane + 64 * i;
      xh[i] = c < d ? ld_elt(x, x_dtype, (size_t)r * x_ld + c) : 0.f;
      sum += xh[i];
    }
    const float mean = wave_sum(sum) / (float)d;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int c = lane + 64 * i;
      xh[i] = c < d ? xh[i] - mean : 0.f;
      sq += xh[i] * xh[i];
    }
    const float rstd = 1.f / sqrtf(wave_sum(sq) / (float)d + eps);
    float m1 = 0.f, m2 = 0.f;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int c = lane + 64 * i;
      xh[i] *= rstd;
      float dn = 0.f;
      if (c < d) {
        const float y = gam[i] * xh[i] + bet[i];
        dn = y > 0.f ? ld_elt(dr, dr_dtype, (size_t)r * dr_ld + c) : 0.f;  // ReLU derivative, strict
        if (dp.threshold > 0) dn = dropout_keep(dp, dp.u0 + r, d, c) ? dn * dp.scale : 0.f;
      }
      dg[i] += dn * xh[i];
      db[i] += dn;
      dxh[i] = dn * gam[i];
      m1 += dxh[i];
      m2 += dxh[i] * xh[i];
    }
    m1 = wave_sum(m1) / (float)d;
    m2 = wave_sum(m2) / (float)d;
    if (out != nullptr) {
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const int c = lane + 64 * i;
        if (c < out_ld) {
          float v = 0.f;
          if (c < d) {
            v = rstd * (dxh[i] - m1 - xh[i] * m2);
            if (res != nullptr) v += ld_elt(res, res_dtype, (size_t)r * res_ld + c);
          }
          st_elt(out, out_dtype, (size_t)r * out_ld + c, v);
        }
      }
    }
  }
  if (wave > 0) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      red[wave - 1][0][lane + 64 * i] = dg[i];
      red[wave - 1][1][lane + 64 * i] = db[i];
    }
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int c = lane + 64 * i;
      if (c < d) {
        partial[((size_t)blockIdx.x * 2 + 0) * d + c] = ((dg[i] + red[0][0][c]) + red[1][0][c]) + red[2][0][c];
        partial[((size_t)blockIdx.x * 2 + 1) * d + c] = ((db[i] + red[0][1][c]) + red[1][1][c]) + red[2][1][c];
      }
    }
  }
}

// One workgroup per 64 entries of the 2 x d sums: 16 wavefronts each add every 16th partial row, then the 16
// slice sums are added in order.
// ---- bf16 rows whose width is 8 x a power of two: LPR lanes per row, 16 bytes per lane, 64 / LPR rows per
// wavefront at a time (the same arithmetic as above, with the loads and stores vectorised)
typedef bf16_t bf16x8_ln __attribute__((ext_vector_type(8)));

template <int LPR>
__device__ inline float group_sum(float v) {
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

template <int LPR>
__global__ __launch_bounds__(256) void ln_relu_vec_kernel(const bf16_t *x, int x_ld, const float *gamma, const float *beta, float eps,
                                                          int64_t M, bf16_t *out, int out_ld, const LnDropout dp) {
  constexpr int RPW = 64 / LPR, d = LPR * 8;
  const int lane = threadIdx.x & 63, sub = lane % LPR, rw = lane / LPR;
  const int64_t w0 = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), nw = (int64_t)gridDim.x * 4;
  float gam[8], bet[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    gam[t] = gamma[sub * 8 + t];
    bet[t] = beta[sub * 8 + t];
  }
  for (int64_t r0 = w0 * RPW; r0 < M; r0 += nw * RPW) {
    const int64_t r = r0 + rw;
    const bool on = r < M;
    const int64_t rr = on ? r : M - 1;  // lanes past the end repeat the last row and do not store
    const bf16x8_ln xv = *reinterpret_cast<const bf16x8_ln *>(x + (size_t)rr * x_ld + sub * 8);
    float v[8], sum = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      v[t] = (float)xv[t];
      sum += v[t];
    }
    const float mean = group_sum<LPR>(sum) / (float)d;
    float sq = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t) sq += (v[t] - mean) * (v[t] - mean);
    const float rstd = 1.f / sqrtf(group_sum<LPR>(sq) / (float)d + eps);
    bf16x8_ln o;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      float y = gam[t] * ((v[t] - mean) * rstd) + bet[t];
      y = y > 0.f ? y : 0.f;
      if (dp.threshold > 0) y = dropout_keep(dp, dp.u0 + rr, d, sub * 8 + t) ? y * dp.scale : 0.f;
      o[t] = (bf16_t)y;
    }
    if (on) *reinterpret_cast<bf16x8_ln *>(out + (size_t)r * out_ld + sub * 8) = o;
  }
}

template <int LPR>
__global__ __launch_bounds__(256) void ln_relu_backward_vec_kernel(const bf16_t *x, int x_ld, const float *gamma, const float *beta,
                                                                   float eps, const bf16_t *dr, int dr_ld, const bf16_t *res, int res_ld,
                                                                   int64_t M, bf16_t *out, int out_ld, float *partial,
                                                                   const LnDropout dp) {
  constexpr int RPW = 64 / LPR, d = LPR * 8;
  __shared__ float red[3][2][LPR * 8];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, sub = lane % LPR, rw = lane / LPR;
  const int64_t w0 = (int64_t)blockIdx.x * 4 + wave, nw = (int64_t)gridDim.x * 4;
  float gam[8], bet[8], dg[8], db[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    gam[t] = gamma[sub * 8 + t];
    bet[t] = beta[sub * 8 + t];
    dg[t] = db[t] = 0.f;
  }
  for (int64_t r0 = w0 * RPW; r0 < M; r0 += nw * RPW) {
    const int64_t r = r0 + rw;
    const bool on = r < M;
    const int64_t rr = on ? r : M - 1;
    const bf16x8_ln xv = *reinterpret_cast<const bf16x8_ln *>(x + (size_t)rr * x_ld + sub * 8);
    const bf16x8_ln dv = *reinterpret_cast<const bf16x8_ln *>(dr + (size_t)rr * dr_ld + sub * 8);
    bf16x8_ln rv;
    if (res != nullptr) rv = *reinterpret_cast<const bf16x8_ln *>(res + (size_t)rr * res_ld + sub * 8);
    float xh[8], dxh[8], sum = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      xh[t] = (float)xv[t];
      sum += xh[t];
    }
    const float mean = group_sum<LPR>(sum) / (float)d;
    float sq = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      xh[t] -= mean;
      sq += xh[t] * xh[t];
    }
    const float rstd = 1.f / sqrtf(group_sum<LPR>(sq) / (float)d + eps);
    float m1 = 0.f, m2 = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      xh[t] *= rstd;
      const float y = gam[t] * xh[t] + bet[t];
      float dn = (on && y > 0.f) ? (float)dv[t] : 0.f;  // ReLU derivative, strict; repeated rows add nothing
      if (dp.threshold > 0) dn = dropout_keep(dp, dp.u0 + rr, d, sub * 8 + t) ? dn * dp.scale : 0.f;
      dg[t] += dn * xh[t];
      db[t] += dn;
      dxh[t] = dn * gam[t];
      m1 += dxh[t];
      m2 += dxh[t] * xh[t];
    }
    m1 = group_sum<LPR>(m1) / (float)d;
    m2 = group_sum<LPR>(m2) / (float)d;
    if (out != nullptr && on) {
      bf16x8_ln o;
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        float v = rstd * (dxh[t] - m1 - xh[t] * m2);
        if (res != nullptr) v += (float)rv[t];
        o[t] = (bf16_t)v;
      }
      *reinterpret_cast<bf16x8_ln *>(out + (size_t)r * out_ld + sub * 8) = o;
    }
  }
  // column sums: over the row groups of the wavefront (fixed order), then over the four wavefronts in LDS
#pragma unroll
  for (int t = 0; t < 8; ++t) {
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1) {
      dg[t] += __shfl_xor(dg[t], o);
      db[t] += __shfl_xor(db[t], o);
    }
  }
  if (wave > 0 && rw == 0) {
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      red[wave - 1][0][sub * 8 + t] = dg[t];
      red[wave - 1][1][sub * 8 + t] = db[t];
    }
  }
  __syncthreads();
  if (wave == 0 && rw == 0) {
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const int c = sub * 8 + t;
      partial[((size_t)blockIdx.x * 2 + 0) * d + c] = ((dg[t] + red[0][0][c]) + red[1][0][c]) + red[2][0][c];
      partial[((size_t)blockIdx.x * 2 + 1) * d + c] = ((db[t] + red[0][1][c]) + red[1][1][c]) + red[2][1][c];
    }
  }
}

// widths served by the vectorised kernels: 64, 128, 256, 512 bf16 columns, 16-byte aligned rows
inline int vec_lanes(int d, int dtype, const void *p, int ld) {
  if (dtype != DT_BF16 || ld % 8 != 0 || (reinterpret_cast<uintptr_t>(p) & 15u)) return 0;
  return (d == 64 || d == 128 || d == 256 || d == 512) ? d / 8 : 0;
}

__global__ __launch_bounds__(1024) void ln_param_reduce_kernel(const float *partial, int n_parts, int d, float *dgamma, float *dbeta) {
  __shared__ float red[16][64];
  const int lane = threadIdx.x & 63, slice = threadIdx.x >> 6;
  const int idx = blockIdx.x * 64 + lane;  // position in [gamma sums | beta sums]
  float s = 0.f;
  if (idx < 2 * d) {
#pragma unroll 8
    for (int w = slice; w < n_parts; w += 16) s += partial[(size_t)w * 2 * d + idx];
  }
  red[slice][lane] = s;
  __syncthreads();
  if (slice == 0 && idx < 2 * d) {
    float t = red[0][lane];
#pragma unroll
    for (int q = 1; q < 16; ++q) t += red[q][lane];
    float *dst = idx < d ? dgamma + idx : dbeta + (idx - d);
    *dst += t;
  }
}

__global__ __launch_bounds__(256) void copy_rows_kernel(const void *src, int src_ld, void *dst, int dst_ld, int64_t M, int d, int dtype) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= M * dst_ld) return;
  const int64_t r = idx / dst_ld;
  const int c = (int)(idx % dst_ld);
  st_elt(dst, dtype, (size_t)idx, c < d ? ld_elt(src, dtype, (size_t)r * src_ld + c) : 0.f);
}

int waves_for(int64_t M, int max_waves) {
  int64_t w = (M + 3) / 4 * 4;  // whole workgroups
  if (w > max_waves) w = max_waves / 4 * 4;
  if (w < 4) w = 4;
  return (int)w;
}

}  // namespace

int launch_ln_relu(const void *x, int x_dtype, int x_ld, const float *gamma, const float *beta, float eps, int64_t M, int d, void *out,
                   int out_dtype, int out_ld, const LnDropout &dp, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  if (d > kLnMaxWidth || out_ld > kLnMaxWidth) return hipErrorInvalidValue;
  const int lpr = (out_dtype == DT_BF16 && out_ld == d && vec_lanes(d, out_dtype, out, out_ld)) ? vec_lanes(d, x_dtype, x, x_ld) : 0;
  if (lpr) {
    const int rpw = 64 / lpr;
    dim3 vgrid((unsigned)(waves_for((M + rpw - 1) / rpw, 16384) / 4));
    const bf16_t *xb = static_cast<const bf16_t *>(x);
    bf16_t *ob = static_cast<bf16_t *>(out);
#define LN_FWD_VEC(L) hipLaunchKernelGGL(ln_relu_vec_kernel<L>, vgrid, dim3(256), 0, s, xb, x_ld, gamma, beta, eps, M, ob, out_ld, dp)
    if (lpr == 8) LN_FWD_VEC(8);
    else if (lpr == 16) LN_FWD_VEC(16);
    else if (lpr == 32) LN_FWD_VEC(32);
    else LN_FWD_VEC(64);
#undef LN_FWD_VEC
    return (int)hipGetLastError();
  }
  const int ni = (std::max(d, out_ld) + 63) / 64;
  dim3 grid((unsigned)(waves_for(M, 16384) / 4));
#define LN_FWD(NI) hipLaunchKernelGGL(ln_relu_kernel<NI>, grid, dim3(256), 0, s, x, x_dtype, x_ld, gamma, beta, eps, M, d, out, out_dtype, out_ld, dp)
  if (ni <= 1) LN_FWD(1);
  else if (ni <= 2) LN_FWD(2);
  else if (ni <= 4) LN_FWD(4);
  else if (ni <= 8) LN_FWD(8);
  else LN_FWD(16);
#undef LN_FWD
  return (int)hipGetLastError();
}

int launch_ln_relu_backward(const void *x, int x_dtype, int x_ld, const float *gamma, const float *beta, float eps, const void *dr,
                            int dr_dtype, int dr_ld, const void *res, int res_dtype, int res_ld, int64_t M, int d, void *out,
                            int out_dtype, int out_ld, float *partial, float *dgamma, float *dbeta, const LnDropout &dp,
                            hipStream_t s) {
  if (M <= 0) return hipSuccess;
  if (d > kLnMaxWidth || (out && out_ld > kLnMaxWidth)) return hipErrorInvalidValue;
  int lpr = vec_lanes(d, x_dtype, x, x_ld);
  if (lpr && (!vec_lanes(d, dr_dtype, dr, dr_ld) || (res && !vec_lanes(d, res_dtype, res, res_ld)) ||
              (out && !vec_lanes(d, out_dtype, out, out_ld))))
    lpr = 0;
  if (lpr) {
    const int rpw = 64 / lpr;
    const int vwaves = waves_for((M + rpw - 1) / rpw, kLnMaxWaves);
    dim3 vgrid((unsigned)(vwaves / 4));
    const bf16_t *xb = static_cast<const bf16_t *>(x), *db = static_cast<const bf16_t *>(dr), *rb = static_cast<const bf16_t *>(res);
    bf16_t *ob = static_cast<bf16_t *>(out);
#define LN_BWD_VEC(L)                                                                                                          \
  hipLaunchKernelGGL(ln_relu_backward_vec_kernel<L>, vgrid, dim3(256), 0, s, xb, x_ld, gamma, beta, eps, db, dr_ld, rb, res_ld, M, ob, \
                     out_ld, partial, dp)
    if (lpr == 8) LN_BWD_VEC(8);
    else if (lpr == 16) LN_BWD_VEC(16);
    else if (lpr == 32) LN_BWD_VEC(32);
    else LN_BWD_VEC(64);
#undef LN_BWD_VEC
    hipError_t ev = hipGetLastError();
    if (ev != hipSuccess) return (int)ev;
    hipLaunchKernelGGL(ln_param_reduce_kernel, dim3((unsigned)((2 * d + 63) / 64)), dim3(1024), 0, s, partial, vwaves / 4, d, dgamma, dbeta);
    return (int)hipGetLastError();
  }
  const int ni = (std::max(d, out ? out_ld : d) + 63) / 64;
  const int waves = waves_for(M, kLnMaxWaves);
  dim3 grid((unsigned)(waves / 4));
#define LN_BWD(NI)                                                                                                              \
  hipLaunchKernelGGL(ln_relu_backward_kernel<NI>, grid, dim3(256), 0, s, x, x_dtype, x_ld, gamma, beta, eps, dr, dr_dtype, dr_ld, res, \
                     res_dtype, res_ld, M, d, out, out_dtype, out_ld, partial, dp)
  if (ni <= 1) LN_BWD(1);
  else if (ni <= 2) LN_BWD(2);
  else if (ni <= 4) LN_BWD(4);
  else if (ni <= 8) LN_BWD(8);
  else LN_BWD(16);
#undef LN_BWD
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return (int)e;
  hipLaunchKernelGGL(ln_param_reduce_kernel, dim3((unsigned)((2 * d + 63) / 64)), dim3(1024), 0, s, partial, waves / 4, d, dgamma, dbeta);
  return (int)hipGetLastError();
}

int launch_copy_rows(const void *src, int src_ld, void *dst, int dst_ld, int64_t M, int d, int dtype, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  hipLaunchKernelGGL(copy_rows_kernel, dim3((unsigned)((M * dst_ld + 255) / 256)), dim3(256), 0, s, src, src_ld, dst, dst_ld, M, d, dtype);
  return (int)hipGetLastError();
}
