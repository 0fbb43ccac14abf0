// Small kernels around the two hot operations: weight staging, the ReLU-derivative mask on
// the upstream gradient, the history copy (Section 3.4, second technique), zero fill, and the
// symmetric normalisation weights of Section 2.1.
#include <algorithm>

#include "common.h"

namespace {

__device__ inline float to_f32(float x) { return x; }
__device__ inline float to_f32(bf16_t x) { return (float)x; }
template <typename T>
__device__ inline T from_f32(float x);
template <>
__device__ inline float from_f32<float>(float x) { return x; }
template <>
__device__ inline bf16_t from_f32<bf16_t>(float x) { return (bf16_t)x; }

// Wt[n][k] = W[k][n] (k < K, else 0; row stride Kp) and Wn[k][n] = W[k][n] (n < N, else 0; row stride Np)
template <typename Tw, typename Tc>
__global__ __launch_bounds__(256) void stage_weights_kernel(const Tw *W, int K, int N, Tc *Wt, int Kp, Tc *Wn, int Np) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx < N * Kp) {
    const int n = idx / Kp, k = idx % Kp;
    Wt[idx] = from_f32<Tc>(k < K ? to_f32(W[(size_t)k * N + n]) : 0.f);
  }
  if (idx < K * Np) {
    const int k = idx / Np, n = idx % Np;
    Wn[idx] = from_f32<Tc>(n < N ? to_f32(W[(size_t)k * N + n]) : 0.f);
  }
}

// 8 elements per thread with 16-byte accesses (d and out_ld multiples of 8, aligned pointers)
template <typename T>
__global__ __launch_bounds__(256) void relu_mask_vec_kernel(const T *g, const T *level, int64_t M, int d, T *out, float scale) {
  typedef T vec_t __attribute__((ext_vector_type(8)));
  const int64_t idx = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
  if (idx >= M * d) return;
  const T *gp = g + idx, *lp = level + idx;
  T *op = out + idx;
  if constexpr (sizeof(T) == 2) {
    const vec_t x = *reinterpret_cast<const vec_t *>(gp), l = *reinterpret_cast<const vec_t *>(lp);
    vec_t r;
#pragma unroll
    for (int t = 0; t < 8; ++t) r[t] = to_f32(l[t]) > 0.f ? from_f32<T>(to_f32(x[t]) * scale) : from_f32<T>(0.f);
    *reinterpret_cast<vec_t *>(op) = r;
  } else {
    typedef T half_t __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const half_t x = *reinterpret_cast<const half_t *>(gp + 4 * h), l = *reinterpret_cast<const half_t *>(lp + 4 * h);
      half_t r;
#pragma unroll
      for (int t = 0; t < 4; ++t) r[t] = to_f32(l[t]) > 0.f ? from_f32<T>(to_f32(x[t]) * scale) : from_f32<T>(0.f);
      *reinterpret_cast<half_t *>(op + 4 * h) = r;
    }
  }
}

// Dropout on rows that a layer has just written: 8 consecutive columns per thread when the row allows it.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void dropout_rows_kernel(T *x, int64_t M, int d, int ld, LnDropout dp) {
  const int per_row = d / VEC;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= M * per_row) return;
  const int64_t r = idx / per_row;
  const int c = (int)(idx % per_row) * VEC;
  typedef T vec_t __attribute__((ext_vector_type(VEC)));
  vec_t *p = reinterpret_cast<vec_t *>(x + r * ld + c);
  vec_t v = *p;
#pragma unroll
  for (int t = 0; t < VEC; ++t) v[t] = dropout_keep(dp, dp.u0 + r, d, c + t) ? from_f32<T>(to_f32(v[t]) * dp.scale) : from_f32<T>(0.f);
  *p = v;
}

template <typename T>
__global__ __launch_bounds__(256) void relu_mask_kernel(const T *g, const T *level, int64_t M, int d, T *out, int out_ld, float scale) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= M * out_ld) return;
  const int64_t m = idx / out_ld;
  const int c = (int)(idx % out_ld);
  float r = 0.f;
  if (c < d && to_f32(level[m * d + c]) > 0.f) r = to_f32(g[m * d + c]) * scale;
  out[idx] = from_f32<T>(r);
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// 16-byte copy with a byte tail.  A workgroup walks contiguous segments (256 KB for large buffers, down to 16 KB for
// small ones so that enough workgroups take part; 2,048 workgroups take the segments round-robin), four 16-byte
// words per thread in flight, loads and stores non-temporal: the bytes are not read
// again soon and need not displace anything in the caches.  Measured against other forms on a 5 GB buffer (read +
// written per second): grid-stride over 4,096 workgroups 4.6 - 4.8 TB/s, over 65,536 workgroups 5.3 TB/s, this form
// 5.4 TB/s, a device-to-device hipMemcpyAsync 4.3 TB/s, a read-only pass 5.3 - 5.7 TB/s, a write-only pass 5.1 TB/s.
__global__ __launch_bounds__(256) void copy_kernel(const u32x4 *src, u32x4 *dst, size_t n16, size_t seg, const uint8_t *tsrc,
                                                   uint8_t *tdst, int tail) {
  const size_t nseg = (n16 + seg - 1) / seg;
  for (size_t sg = blockIdx.x; sg < nseg; sg += gridDim.x) {
    const size_t b = sg * seg, e = b + seg < n16 ? b + seg : n16;
    size_t i = b + threadIdx.x;
    for (; i + 3 * 256 < e; i += 4 * 256) {
      u32x4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(src + i + u * 256);
#pragma unroll
      for (int u = 0; u < 4; ++u) __builtin_nontemporal_store(v[u], dst + i + u * 256);
    }
    for (; i < e; i += 256) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
  }
  if (blockIdx.x == 0 && (int)threadIdx.x < tail) tdst[threadIdx.x] = tsrc[threadIdx.x];
}

__global__ __launch_bounds__(256) void fill_zero_kernel(u32x4 *dst, size_t n16, uint8_t *tdst, int tail) {
  const size_t stride = (size_t)gridDim.x * 256;
  const u32x4 z = {0u, 0u, 0u, 0u};
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = z;
  if (blockIdx.x == 0 && (int)threadIdx.x < tail) tdst[threadIdx.x] = 0;
}

// One wave per sparse row: val[e] = 1 / sqrt(len(row) * len(other endpoint)), lengths taken from
// len_ptr (the CSR row pointer of A + I), computed in fp64 and rounded once to fp32.
__global__ __launch_bounds__(256) void gcn_norm_kernel(const int64_t *ptr, const uint32_t *pidx, int vbits,
                                                       const int64_t *len_ptr, int64_t n, float *val) {
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= n) return;
  const int lane = threadIdx.x & 63;
  const uint32_t vmask = (1u << vbits) - 1u;
  const double dv = (double)(len_ptr[row + 1] - len_ptr[row]);
  for (int64_t e = ptr[row] + lane; e < ptr[row + 1]; e += 64) {
    const int64_t u = pidx[e] & vmask;
    const double du = (double)(len_ptr[u + 1] - len_ptr[u]);
    val[e] = (float)(1.0 / sqrt(dv * du));
  }
}

}  // namespace

int launch_stage_weights(const void *W, int w_dtype, int K, int N, void *Wt, int Kp, void *Wn, int Np, hipStream_t s) {
  const int total = (N * Kp > K * Np) ? N * Kp : K * Np;
  dim3 grid((total + 255) / 256);
  if (w_dtype == DT_BF16)
    hipLaunchKernelGGL((stage_weights_kernel<bf16_t, bf16_t>), grid, dim3(256), 0, s, static_cast<const bf16_t *>(W), K, N,
                       static_cast<bf16_t *>(Wt), Kp, static_cast<bf16_t *>(Wn), Np);
  else
    hipLaunchKernelGGL((stage_weights_kernel<float, float>), grid, dim3(256), 0, s, static_cast<const float *>(W), K, N,
                       static_cast<float *>(Wt), Kp, static_cast<float *>(Wn), Np);
  return (int)hipGetLastError();
}

int launch_dropout_rows(void *x, int dtype, int64_t M, int d, int ld, const LnDropout &dp, hipStream_t s) {
  if (M <= 0 || d <= 0 || dp.threshold == 0) return hipSuccess;
  const bool vec = d % 8 == 0 && ld % 8 == 0 && (reinterpret_cast<uintptr_t>(x) & 15u) == 0 && dtype == DT_BF16;
  const int64_t threads = vec ? M * (d / 8) : M * d;
  dim3 grid((unsigned)((threads + 255) / 256));
  if (dtype == DT_BF16) {
    if (vec)
      hipLaunchKernelGGL((dropout_rows_kernel<bf16_t, 8>), grid, dim3(256), 0, s, static_cast<bf16_t *>(x), M, d, ld, dp);
    else
      hipLaunchKernelGGL((dropout_rows_kernel<bf16_t, 1>), grid, dim3(256), 0, s, static_cast<bf16_t *>(x), M, d, ld, dp);
  } else {
    hipLaunchKernelGGL((dropout_rows_kernel<float, 1>), grid, dim3(256), 0, s, static_cast<float *>(x), M, d, ld, dp);
  }
  return (int)hipGetLastError();
}

int launch_relu_mask(const void *g, const void *level, int dtype, int64_t M, int d, void *out, int out_ld, float scale,
                     hipStream_t s) {
  if (M <= 0) return hipSuccess;
  const auto al = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
  if (d % 8 == 0 && out_ld == d && al(g) && al(level) && al(out)) {
    dim3 gv((unsigned)((M * d / 8 + 255) / 256));
    if (dtype == DT_BF16)
      hipLaunchKernelGGL(relu_mask_vec_kernel<bf16_t>, gv, dim3(256), 0, s, static_cast<const bf16_t *>(g),
                         static_cast<const bf16_t *>(level), M, d, static_cast<bf16_t *>(out), scale);
    else
      hipLaunchKernelGGL(relu_mask_vec_kernel<float>, gv, dim3(256), 0, s, static_cast<const float *>(g),
                         static_cast<const float *>(level), M, d, static_cast<float *>(out), scale);
    return (int)hipGetLastError();
  }
  const int64_t total = M * out_ld;
  dim3 grid((unsigned)((total + 255) / 256));
  if (dtype == DT_BF16)
    hipLaunchKernelGGL(relu_mask_kernel<bf16_t>, grid, dim3(256), 0, s, static_cast<const bf16_t *>(g),
                       static_cast<const bf16_t *>(level), M, d, static_cast<bf16_t *>(out), out_ld, scale);
  else
    hipLaunchKernelGGL(relu_mask_kernel<float>, grid, dim3(256), 0, s, static_cast<const float *>(g),
                       static_cast<const float *>(level), M, d, static_cast<float *>(out), out_ld, scale);
  return (int)hipGetLastError();
}

static unsigned stream_grid(size_t n16) {
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 256 * 16) blocks = 256 * 16;  // 16 blocks per CU, grid-stride beyond that
  if (blocks == 0) blocks = 1;
  return (unsigned)blocks;
}

// ---- what the memory system gives a row gather (diagnostic) --------------------------------------------
// Every 16-lane group reads whole rows of row_bytes (16 bytes per lane and step) at pseudo-random row numbers,
// eight rows in flight per group, and folds what it read into one word so that no load can be dropped.  A share
// of the draws goes to the first hot_rows rows (a power-law graph's hubs); the others are uniform over the table.
namespace {
__device__ inline uint32_t mix32(uint32_t x) {
  x ^= x >> 16;
  x *= 0x7feb352du;
  x ^= x >> 15;
  x *= 0x846ca68bu;
  return x ^ (x >> 16);
}

template <int MODE>  // 0: plain loads, 1: non-temporal loads, 2: plain loads, hot rows scattered, 3: non-temporal loads for the cold draws only
__global__ __launch_bounds__(256) void gather_probe_kernel(const u32x4 *table, uint32_t n_rows, int row_vecs, int rows_per_group,
                                                           uint32_t hot_rows, uint32_t hot_threshold, uint32_t seed, uint32_t *sink) {
  const uint32_t group = (blockIdx.x * 256u + threadIdx.x) >> 4;
  const int lig = threadIdx.x & 15;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (int i = 0; i < rows_per_group; i += 8) {
    u32x4 x[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const uint32_t h = mix32(seed + group * 0x9e3779b9u + (uint32_t)(i + u));
      const uint32_t pick = mix32(h ^ 0x85ebca6bu);
      uint32_t row = (pick < hot_threshold) ? h % hot_rows : h % n_rows;
      if (MODE == 2 && pick < hot_threshold) row *= n_rows / hot_rows;  // the hot rows spread evenly over the table
      const u32x4 *p = table + (size_t)row * row_vecs + lig;
      const bool nt = MODE == 1 || (MODE == 3 && pick >= hot_threshold);
      x[u] = nt ? __builtin_nontemporal_load(p) : p[0];
      for (int v = 16; v < row_vecs; v += 16) {
        const u32x4 y = nt ? __builtin_nontemporal_load(p + v) : p[v];
        x[u] ^= y;
      }
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= x[u];
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345677u) sink[0] = group;  // practically never true; keeps the loads alive
}

}  // namespace

// Times n_launches launches of the probe on `stream` with HIP events and reports bytes gathered per second.
// table: DEVICE, n_rows rows of row_bytes (a multiple of 256, at most 4096); sink: DEVICE, 4 bytes.
extern "C" int gnnstage_debug_gather_rate(const void *table, int64_t n_rows, int32_t row_bytes, int64_t gathers_per_launch,
                                          int32_t n_launches, int64_t hot_rows, double hot_share, int32_t mode, uint32_t seed,
                                          void *sink, void *hip_stream, double *bytes_per_second) {
  if (!table || !sink || !bytes_per_second || n_rows < 1 || n_rows > 0xffffffffll || row_bytes < 256 || row_bytes > 4096 ||
      row_bytes % 256 != 0 || gathers_per_launch < 1 || n_launches < 1 || hot_rows < 0 || hot_rows > n_rows ||
      !(hot_share >= 0.0 && hot_share <= 1.0) || (hot_share > 0.0 && hot_rows < 1) || mode < 0 || mode > 3)
    return -1;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int blocks = 256 * 8;  // eight workgroups of four waves per compute unit: full occupancy
  const int64_t groups = (int64_t)blocks * 16;
  int64_t per_group = (gathers_per_launch + groups - 1) / groups;
  per_group = (per_group + 7) / 8 * 8;
  if (per_group > (1 << 24)) return -1;
  const uint32_t thr = hot_share >= 1.0 ? 0xffffffffu : (uint32_t)(hot_share * 4294967296.0);
  hipEvent_t a = nullptr, b = nullptr;
  if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return -5;
  auto launch = [&](uint32_t sd) {
    const u32x4 *t = static_cast<const u32x4 *>(table);
    const uint32_t hr = (uint32_t)std::max<int64_t>(hot_rows, 1);
    uint32_t *sk = static_cast<uint32_t *>(sink);
    if (mode == 3)
      hipLaunchKernelGGL(gather_probe_kernel<3>, dim3(blocks), dim3(256), 0, s, t, (uint32_t)n_rows, row_bytes / 16, (int)per_group, hr, thr, sd, sk);
    else if (mode == 2)
      hipLaunchKernelGGL(gather_probe_kernel<2>, dim3(blocks), dim3(256), 0, s, t, (uint32_t)n_rows, row_bytes / 16, (int)per_group, hr, thr, sd, sk);
    else if (mode == 1)
      hipLaunchKernelGGL(gather_probe_kernel<1>, dim3(blocks), dim3(256), 0, s, t, (uint32_t)n_rows, row_bytes / 16, (int)per_group, hr, thr, sd, sk);
    else
      hipLaunchKernelGGL(gather_probe_kernel<0>, dim3(blocks), dim3(256), 0, s, t, (uint32_t)n_rows, row_bytes / 16, (int)per_group, hr, thr, sd, sk);
  };
  launch(seed);  // warm-up
  (void)hipEventRecord(a, s);
  for (int i = 0; i < n_launches; ++i) launch(seed + 1u + (uint32_t)i);
  (void)hipEventRecord(b, s);
  float ms = 0.f;
  const bool ok = hipEventSynchronize(b) == hipSuccess && hipEventElapsedTime(&ms, a, b) == hipSuccess && hipGetLastError() == hipSuccess;
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  if (!ok || !(ms > 0.f)) return -5;
  *bytes_per_second = (double)per_group * (double)groups * (double)row_bytes * n_launches / ((double)ms * 1e-3);
  return 0;
}

int launch_copy(const void *src, void *dst, size_t bytes, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  const size_t n16 = bytes / 16;
  const int tail = (int)(bytes % 16);
  // segment length in 16-byte words: a 2,048th of the buffer, in steps of 16 KB, between 16 KB and 256 KB
  size_t seg = ((n16 / 2048 + 1023) / 1024) * 1024;
  seg = seg < 1024 ? 1024 : seg > 16384 ? 16384 : seg;
  const size_t nseg = (n16 + seg - 1) / seg;
  const unsigned grid = (unsigned)(nseg < 1 ? 1 : nseg > 2048 ? 2048 : nseg);
  hipLaunchKernelGGL(copy_kernel, dim3(grid), dim3(256), 0, s, static_cast<const u32x4 *>(src),
                     static_cast<u32x4 *>(dst), n16, seg, static_cast<const uint8_t *>(src) + n16 * 16,
                     static_cast<uint8_t *>(dst) + n16 * 16, tail);
  return (int)hipGetLastError();
}

int launch_fill_zero(void *dst, size_t bytes, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  const size_t n16 = bytes / 16;
  const int tail = (int)(bytes % 16);
  hipLaunchKernelGGL(fill_zero_kernel, dim3(stream_grid(n16)), dim3(256), 0, s, static_cast<u32x4 *>(dst), n16,
                     static_cast<uint8_t *>(dst) + n16 * 16, tail);
  return (int)hipGetLastError();
}

int launch_gcn_norm(const int64_t *ptr, const uint32_t *pidx, int vbits, const int64_t *len_ptr, int64_t n, float *val,
                    hipStream_t s) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(gcn_norm_kernel, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, s, ptr, pidx, vbits, len_ptr, n, val);
  return (int)hipGetLastError();
}
