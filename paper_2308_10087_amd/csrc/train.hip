// The epoch loop of Algorithm 1 around stage handles: chunk shuffling and the history refresh period
// (Section 3.4, techniques 1 and 2), a linear softmax cross-entropy head, the weight update (Algorithm 1's
// last line, or Adam as in Section 5).  The stages do the heavy work through their public entry points; the
// head reuses the library's dense products.
#include <hip/hip_runtime.h>
#include "guard.h"
#include <memory>

#include <algorithm>
#include <cmath>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/gnntrain.h"
#include "common.h"

namespace {

constexpr int kMaxSplits = 256;  // split-reduction scratch of the weight-gradient product
constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;

std::string g_create_error;

inline uint64_t splitmix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

inline int round_up(int x, int m) { return (x + m - 1) / m * m; }
inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

__device__ inline void store_elt(void *p, int dtype, size_t idx, float v) {
  if (dtype == DT_BF16)
    static_cast<bf16_t *>(p)[idx] = (bf16_t)v;
  else
    static_cast<float *>(p)[idx] = v;
}

// One wavefront per vertex: maximum, sum of exponentials, then the gradient row.
__global__ __launch_bounds__(256) void softmax_xent_kernel(const float *logits, int ld, const float *bias, const int32_t *labels,
                                                           const uint8_t *mask, int64_t rows, int C, float inv_n, void *dlogits,
                                                           int dl_dtype, int dl_ld, float *row_loss) {
  const int lane = threadIdx.x & 63;
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;  // whole wave
  const bool labelled = mask == nullptr || mask[r] != 0;
  if (!labelled) {
    for (int c = lane; c < dl_ld; c += 64) store_elt(dlogits, dl_dtype, (size_t)r * dl_ld + c, 0.f);
    if (lane == 0) row_loss[r] = 0.f;
    return;
  }
  const float *z = logits + (size_t)r * ld;
  const int label = labels[r];
  float mx = -INFINITY;
  for (int c = lane; c < C; c += 64) mx = fmaxf(mx, z[c] + (bias ? bias[c] : 0.f));
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
  // the label's own term is kept apart: softmax_label - 1 = -(sum of the others) / sum has no cancellation,
  // and a confident row's loss is log1p(others / own)
  float others = 0.f;
  for (int c = lane; c < C; c += 64)
    if (c != label) others += expf(z[c] + (bias ? bias[c] : 0.f) - mx);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) others += __shfl_xor(others, o);
  const float zl = z[label] + (bias ? bias[label] : 0.f) - mx;
  const float own = expf(zl);
  const float sum = others + own;
  const float inv_sum = 1.f / sum;
  for (int c = lane; c < dl_ld; c += 64) {
    float g = 0.f;
    if (c < C) {
      const float p = expf(z[c] + (bias ? bias[c] : 0.f) - mx) * inv_sum;
      g = (c == label ? -others * inv_sum : p) * inv_n;
    }
    store_elt(dlogits, dl_dtype, (size_t)r * dl_ld + c, g);
  }
  if (lane == 0) row_loss[r] = own > 0.5f * sum ? log1pf(others / own) : logf(sum) - zl;
}

// Fixed-order sum: block b adds its contiguous slice (thread-strided, then an LDS tree), a second launch
// adds the block sums the same way.
__global__ __launch_bounds__(256) void sum_slices_kernel(const float *x, int64_t n, int64_t per_block, float scale, float *out) {
  __shared__ float red[256];
  const int64_t b0 = (int64_t)blockIdx.x * per_block;
  const int64_t b1 = b0 + per_block < n ? b0 + per_block : n;
  float s = 0.f;
  for (int64_t i = b0 + threadIdx.x; i < b1; i += 256) s += x[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[blockIdx.x] = red[0] * scale;
}

__global__ __launch_bounds__(256) void adam_kernel(float *p, const float *g, float *m, float *v, void *compute, int compute_dtype,
                                                   int64_t n, float lr, float b1, float b2, float eps, float wd, float c1, float c2) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const float pi = p[i];
  const float gi = g[i] + wd * pi;
  const float mi = b1 * m[i] + (1.f - b1) * gi;
  const float vi = b2 * v[i] + (1.f - b2) * gi * gi;
  m[i] = mi;
  v[i] = vi;
  const float pn = pi - lr * (mi * c1) / (sqrtf(vi * c2) + eps);
  p[i] = pn;
  if (compute) store_elt(compute, compute_dtype, (size_t)i, pn);
}

__global__ __launch_bounds__(256) void sgd_kernel(float *p, const float *g, void *compute, int compute_dtype, int64_t n, float lr,
                                                  float wd) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const float pi = p[i];
  const float pn = pi - lr * (g[i] + wd * pi);
  p[i] = pn;
  if (compute) store_elt(compute, compute_dtype, (size_t)i, pn);
}

struct Layout {
  size_t m = 0, v = 0, logits = 0, dlogits = 0, dtop = 0, row_loss = 0, scratch = 0, loss = 0, Wt = 0, Wn = 0, gemm_partial = 0,
         bias_partial = 0, total = 0;
};

struct Dims {
  int64_t n = 0, max_rows = 0, n_param_elems = 0;
  int K = 0, d_top = 0, C = 0, Cp = 0, Kp = 0, dtype = 0, elt = 4;
};

bool read_dims(const gnntrain_desc *d, Dims &x, std::string &err) {
  if (!d) { err = "descriptor is NULL"; return false; }
  if (d->n_stages <= 0 || !d->stages) { err = "no stages"; return false; }
  for (int s = 0; s < d->n_stages; ++s)
    if (!d->stages[s]) { err = "a stage handle is NULL"; return false; }
  if (d->n_classes <= 0 || d->n_classes > 65536) { err = "n_classes must be in [1, 65536]"; return false; }
  if (d->n_params < 0 || (d->n_params > 0 && !d->params)) { err = "params is NULL"; return false; }
  if (d->optimizer != GNNTRAIN_SGD && d->optimizer != GNNTRAIN_ADAM) { err = "unknown optimizer"; return false; }
  if (d->alpha_hist < 1) { err = "alpha_hist must be at least 1"; return false; }
  const gnnstage_t *last = d->stages[d->n_stages - 1];
  x.n = gnnstage_query(last, GNNSTAGE_Q_VERTICES, 0);
  x.K = (int)gnnstage_query(last, GNNSTAGE_Q_CHUNKS, 0);
  const int L = (int)gnnstage_query(last, GNNSTAGE_Q_LAYERS, 0);
  x.d_top = (int)gnnstage_query(last, GNNSTAGE_Q_WIDTH, L);
  x.dtype = (int)gnnstage_query(last, GNNSTAGE_Q_DTYPE, 0);
  x.elt = x.dtype == GNNSTAGE_BF16 ? 2 : 4;
  x.C = d->n_classes;
  x.Cp = round_up(x.C, 8);
  x.Kp = round_up(x.d_top, 8);
  x.max_rows = 0;
  for (int c = 0; c < x.K; ++c)
    x.max_rows = std::max<int64_t>(x.max_rows, gnnstage_query(last, GNNSTAGE_Q_CHUNK_PTR, c + 1) - gnnstage_query(last, GNNSTAGE_Q_CHUNK_PTR, c));
  x.n_param_elems = 0;
  for (int i = 0; i < d->n_params; ++i) {
    const gnntrain_param &p = d->params[i];
    if (!p.master || !p.grad || p.count <= 0) { err = "a parameter has a NULL pointer or no elements"; return false; }
    if (p.compute_dtype != GNNSTAGE_F32 && p.compute_dtype != GNNSTAGE_BF16) { err = "unknown parameter dtype"; return false; }
    x.n_param_elems += (p.count + 63) / 64 * 64;
  }
  return true;
}

Layout make_layout(const gnntrain_desc *d, const Dims &x) {
  Layout l;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off = align256(off + bytes);
    return at;
  };
  const size_t moments = d->optimizer == GNNTRAIN_ADAM ? sizeof(float) * (size_t)x.n_param_elems : 0;
  l.m = take(moments);
  l.v = take(moments);
  l.logits = take(sizeof(float) * (size_t)x.max_rows * x.Cp);
  l.dlogits = take((size_t)x.elt * x.n * x.Cp);
  l.dtop = take((size_t)x.elt * x.max_rows * x.d_top);
  l.row_loss = take(sizeof(float) * (size_t)x.n);
  l.scratch = take(sizeof(float) * 1024);
  l.loss = take(256);
  l.Wt = take((size_t)x.elt * x.C * x.Kp);
  l.Wn = take((size_t)x.elt * x.d_top * x.Cp);
  l.gemm_partial = take(sizeof(float) * (size_t)kMaxSplits * x.d_top * x.C);
  l.bias_partial = take(sizeof(float) * (size_t)kMaxSplits * x.Cp);
  l.total = off;
  return l;
}

}  // namespace

struct gnntrain {
  Dims x;
  Layout lay;
  std::vector<gnnstage_t *> stages;
  std::vector<int64_t> chunk_ptr;
  std::vector<gnntrain_param> params;
  std::vector<size_t> moment_off;  // element offset of every parameter inside m / v
  const void *top = nullptr;
  const void *head_W = nullptr;
  const float *head_b = nullptr;
  float *head_dW = nullptr, *head_db = nullptr;
  const int32_t *labels = nullptr;
  const uint8_t *mask = nullptr;
  int64_t n_train = 0;
  int optimizer = 0, shuffle = 0, alpha_hist = 1, history_swap = 0;
  float lr = 0, beta1 = 0, beta2 = 0, eps = 0, wd = 0;
  uint64_t seed = 0;
  int64_t step = 0;
  char *ws = nullptr;
  std::vector<int32_t> order;
  std::string err;
  template <typename T>
  T *at(size_t off) const { return reinterpret_cast<T *>(ws + off); }
};

namespace {

int fail(gnntrain *tr, int code, const std::string &msg) {
  tr->err = msg;
  return code;
}

#define TRAIN_HIP(tr, expr)                                                                    \
  do {                                                                                         \
    const int e_ = (int)(expr);                                                                \
    if (e_ != 0) return fail(tr, GNNSTAGE_EHIP, std::string(#expr) + ": " + hipGetErrorString((hipError_t)e_)); \
  } while (0)

#define TRAIN_STAGE(tr, s, expr)                                                               \
  do {                                                                                         \
    const int e_ = (expr);                                                                     \
    if (e_ != GNNSTAGE_OK) return fail(tr, e_, std::string("stage: ") + gnnstage_last_error(tr->stages[s])); \
  } while (0)

int launch_sum(const float *x, int64_t n, float scale, float *scratch, float *out, hipStream_t s) {
  int64_t blocks = (n + 4095) / 4096;
  if (blocks > 1024) blocks = 1024;
  if (blocks < 1) blocks = 1;
  const int64_t per = (n + blocks - 1) / blocks;
  hipLaunchKernelGGL(sum_slices_kernel, dim3((unsigned)blocks), dim3(256), 0, s, x, n, per, 1.f, scratch);
  hipLaunchKernelGGL(sum_slices_kernel, dim3(1), dim3(256), 0, s, scratch, blocks, blocks, scale, out);
  return (int)hipGetLastError();
}

}  // namespace

extern "C" int gnntrain_chunk_order(uint64_t seed, int64_t epoch, int32_t n_chunks, int32_t shuffle, int32_t *order) try {
  if (!order || n_chunks <= 0 || epoch < 0) return GNNSTAGE_EINVAL;
  for (int i = 0; i < n_chunks; ++i) order[i] = i;
  if (!shuffle) return GNNSTAGE_OK;
  const uint64_t start = seed + (uint64_t)(epoch + 1) * kGolden;
  uint64_t draw = 0;
  for (int i = n_chunks - 1; i > 0; --i) {
    ++draw;
    const uint64_t r = splitmix64(start + draw * kGolden);
    const int j = (int)(r % (uint64_t)(i + 1));
    const int32_t t = order[i];
    order[i] = order[j];
    order[j] = t;
  }
  return GNNSTAGE_OK;
}
GNNSTAGE_GUARD_INT

extern "C" int gnntrain_softmax_xent(const float *logits, int32_t ld, const float *bias, const int32_t *labels, const uint8_t *mask,
                                     int64_t rows, int32_t n_classes, float inv_n_train, void *dlogits, int32_t dl_dtype,
                                     int32_t dl_ld, float *row_loss, void *hip_stream) {
  if (rows < 0 || n_classes <= 0 || ld < n_classes || dl_ld < n_classes) return GNNSTAGE_EINVAL;
  if (dl_dtype != GNNSTAGE_F32 && dl_dtype != GNNSTAGE_BF16) return GNNSTAGE_EINVAL;
  if (rows == 0) return GNNSTAGE_OK;
  if (!logits || !labels || !dlogits || !row_loss) return GNNSTAGE_EINVAL;
  hipLaunchKernelGGL(softmax_xent_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, static_cast<hipStream_t>(hip_stream), logits,
                     ld, bias, labels, mask, rows, n_classes, inv_n_train, dlogits, dl_dtype, dl_ld, row_loss);
  return hipGetLastError() == hipSuccess ? GNNSTAGE_OK : GNNSTAGE_EHIP;
}

extern "C" int gnntrain_sum(const float *x, int64_t n, float scale, float *scratch, float *out, void *hip_stream) {
  if (n < 0 || !scratch || !out || (n > 0 && !x)) return GNNSTAGE_EINVAL;
  return launch_sum(x, n, scale, scratch, out, static_cast<hipStream_t>(hip_stream)) == 0 ? GNNSTAGE_OK : GNNSTAGE_EHIP;
}

// ---- the same sum for callers that cannot allocate -----------------------------------------------------
// The block sums go to a file-scope device array instead of a buffer the caller brings.  Every GPU holds its own
// copy of the array at its own address; host code never uses the array's name (a host-side stand-in, not a
// device address) but the address hipGetSymbolAddress reports for the device that is current, looked up once per
// device and kept.
constexpr int kSumStaticSlots = 1024;  // block sums of one call: the kernels never use more blocks than this
static __device__ __align__(256) float scratch[kSumStaticSlots];
namespace {
constexpr int kMaxDevices = 64;
float *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// device address of `scratch` on the current device; nullptr (with err set) when it cannot be had
float *static_scratch(std::string &err) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) {
    err = std::string("hipGetDevice: ") + hipGetErrorString(e);
    return nullptr;
  }
  if (dev < 0 || dev >= kMaxDevices) {
    err = "device index beyond the per-device table of the static scratch array";
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void *ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || ptr == nullptr) {
      err = std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e);
      return nullptr;
    }
    g_scratch_ptr[dev] = static_cast<float *>(ptr);
  }
  return g_scratch_ptr[dev];
}
}  // namespace

extern "C" int gnntrain_sum_static(const float *x, int64_t n, float scale, float *out, void *hip_stream) {
  if (n < 0 || !out || (n > 0 && !x)) {
    g_create_error = "gnntrain_sum_static: n is negative or a pointer is NULL";
    return GNNSTAGE_EINVAL;
  }
  if (n > GNNTRAIN_SUM_STATIC_MAX_N) {
    g_create_error = "gnntrain_sum_static: n exceeds GNNTRAIN_SUM_STATIC_MAX_N (2^31 - 1 elements)";
    return GNNSTAGE_ENOTSUP;
  }
  std::string err;
  float *ptr = static_scratch(err);
  if (ptr == nullptr) {
    g_create_error = err;
    return GNNSTAGE_EHIP;
  }
  // Nothing in the array has to start at zero: the first launch writes every slot the second one reads.
  return launch_sum(x, n, scale, ptr, out, static_cast<hipStream_t>(hip_stream)) == 0 ? GNNSTAGE_OK : GNNSTAGE_EHIP;
}

extern "C" int gnntrain_adam_step(float *p, const float *g, float *m, float *v, void *compute, int32_t compute_dtype, int64_t count,
                                  float lr, float beta1, float beta2, float eps, float weight_decay, int64_t t, void *hip_stream) {
  if (count < 0 || t < 1) return GNNSTAGE_EINVAL;
  if (count == 0) return GNNSTAGE_OK;
  if (!p || !g || !m || !v) return GNNSTAGE_EINVAL;
  if (compute_dtype != GNNSTAGE_F32 && compute_dtype != GNNSTAGE_BF16) return GNNSTAGE_EINVAL;
  if (compute == p) compute = nullptr;
  // bias corrections 1 / (1 - beta^t), formed in double on the host
  const float c1 = (float)(1.0 / (1.0 - std::pow((double)beta1, (double)t)));
  const float c2 = (float)(1.0 / (1.0 - std::pow((double)beta2, (double)t)));
  hipLaunchKernelGGL(adam_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(hip_stream), p, g, m, v,
                     compute, compute_dtype, count, lr, beta1, beta2, eps, weight_decay, c1, c2);
  return hipGetLastError() == hipSuccess ? GNNSTAGE_OK : GNNSTAGE_EHIP;
}

extern "C" int gnntrain_sgd_step(float *p, const float *g, void *compute, int32_t compute_dtype, int64_t count, float lr,
                                 float weight_decay, void *hip_stream) {
  if (count < 0) return GNNSTAGE_EINVAL;
  if (count == 0) return GNNSTAGE_OK;
  if (!p || !g) return GNNSTAGE_EINVAL;
  if (compute_dtype != GNNSTAGE_F32 && compute_dtype != GNNSTAGE_BF16) return GNNSTAGE_EINVAL;
  if (compute == p) compute = nullptr;
  hipLaunchKernelGGL(sgd_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(hip_stream), p, g,
                     compute, compute_dtype, count, lr, weight_decay);
  return hipGetLastError() == hipSuccess ? GNNSTAGE_OK : GNNSTAGE_EHIP;
}

extern "C" size_t gnntrain_workspace_size(const gnntrain_desc *desc) try {
  Dims x;
  std::string err;
  if (!read_dims(desc, x, err)) return 0;
  return make_layout(desc, x).total;
}
GNNSTAGE_GUARD_SIZE

extern "C" const char *gnntrain_last_error(const gnntrain_t *tr) { return tr ? tr->err.c_str() : g_create_error.c_str(); }

extern "C" int gnntrain_create(const gnntrain_desc *d, gnntrain_t **out) try {
  if (out) *out = nullptr;
  auto bad = [&](int code, const std::string &msg) {
    g_create_error = msg;
    return code;
  };
  if (!out) return bad(GNNSTAGE_EINVAL, "out is NULL");
  Dims x;
  std::string err;
  if (!read_dims(d, x, err)) return bad(GNNSTAGE_EINVAL, err);
  if (!d->head_W || !d->head_b || !d->head_dW || !d->head_db || !d->labels) return bad(GNNSTAGE_EINVAL, "head pointers and labels must not be NULL");
  const Layout lay = make_layout(d, x);
  if (!d->workspace || (reinterpret_cast<uintptr_t>(d->workspace) & 255u)) return bad(GNNSTAGE_EINVAL, "workspace must be 256-byte aligned");
  if (d->workspace_bytes < lay.total) return bad(GNNSTAGE_ENOMEM, "workspace smaller than gnntrain_workspace_size()");
  // the stages must describe one model: same vertices and chunks, level buffers chained, gradients too
  for (int s = 0; s < d->n_stages; ++s) {
    const gnnstage_t *st = d->stages[s];
    if (gnnstage_query(st, GNNSTAGE_Q_VERTICES, 0) != x.n || gnnstage_query(st, GNNSTAGE_Q_CHUNKS, 0) != x.K)
      return bad(GNNSTAGE_EINVAL, "stages differ in vertex or chunk count");
    for (int c = 0; c <= x.K; ++c)
      if (gnnstage_query(st, GNNSTAGE_Q_CHUNK_PTR, c) != gnnstage_query(d->stages[0], GNNSTAGE_Q_CHUNK_PTR, c))
        return bad(GNNSTAGE_EINVAL, "stages differ in chunk boundaries");
    if (s > 0) {
      const gnnstage_t *prev = d->stages[s - 1];
      const int Lp = (int)gnnstage_query(prev, GNNSTAGE_Q_LAYERS, 0);
      if (gnnstage_buffer(st, GNNSTAGE_B_CUR, 0) != gnnstage_buffer(prev, GNNSTAGE_B_CUR, Lp))
        return bad(GNNSTAGE_EINVAL, "level 0 of a stage must be the last level of the stage before it (same device buffer)");
      if (gnnstage_query(st, GNNSTAGE_Q_WIDTH, 0) != gnnstage_query(prev, GNNSTAGE_Q_WIDTH, Lp))
        return bad(GNNSTAGE_EINVAL, "widths of chained levels differ");
      if (gnnstage_query(st, GNNSTAGE_Q_DTYPE, 0) != gnnstage_query(prev, GNNSTAGE_Q_DTYPE, 0) ||
          gnnstage_query(st, GNNSTAGE_Q_LEVEL0_F32, 0) != 0)
        return bad(GNNSTAGE_EINVAL, "chained stages must share the level dtype");
      if (!gnnstage_buffer(st, GNNSTAGE_B_GRAD_IN, 0))
        return bad(GNNSTAGE_EINVAL, "every stage after the first must be created with need_input_grad and a grad_in buffer");
    }
  }
  // labels are checked once, on the host
  std::vector<int32_t> lab((size_t)x.n);
  if (hipMemcpy(lab.data(), d->labels, sizeof(int32_t) * (size_t)x.n, hipMemcpyDeviceToHost) != hipSuccess)
    return bad(GNNSTAGE_EHIP, "reading the labels failed");
  for (int64_t i = 0; i < x.n; ++i)
    if (lab[(size_t)i] < 0 || lab[(size_t)i] >= x.C) return bad(GNNSTAGE_EINVAL, "a label is outside [0, n_classes)");
  int64_t n_train = x.n;
  if (d->train_mask) {
    std::vector<uint8_t> mk((size_t)x.n);
    if (hipMemcpy(mk.data(), d->train_mask, (size_t)x.n, hipMemcpyDeviceToHost) != hipSuccess)
      return bad(GNNSTAGE_EHIP, "reading the training mask failed");
    n_train = 0;
    for (int64_t i = 0; i < x.n; ++i) n_train += mk[(size_t)i] != 0;
  }
  if (n_train <= 0) return bad(GNNSTAGE_EINVAL, "no labelled vertex");

  std::unique_ptr<gnntrain> holder(new gnntrain());  // freed on an early return, and when something below throws
  gnntrain *tr = holder.get();
  tr->x = x;
  tr->lay = lay;
  tr->stages.assign(d->stages, d->stages + d->n_stages);
  tr->chunk_ptr.resize((size_t)x.K + 1);
  for (int c = 0; c <= x.K; ++c) tr->chunk_ptr[(size_t)c] = gnnstage_query(d->stages[0], GNNSTAGE_Q_CHUNK_PTR, c);
  tr->params.assign(d->params, d->params + d->n_params);
  size_t off = 0;
  for (const gnntrain_param &p : tr->params) {
    tr->moment_off.push_back(off);
    off += (size_t)((p.count + 63) / 64 * 64);
  }
  const gnnstage_t *last = tr->stages.back();
  tr->top = gnnstage_buffer(last, GNNSTAGE_B_CUR, (int)gnnstage_query(last, GNNSTAGE_Q_LAYERS, 0));
  tr->head_W = d->head_W;
  tr->head_b = d->head_b;
  tr->head_dW = d->head_dW;
  tr->head_db = d->head_db;
  tr->labels = d->labels;
  tr->mask = d->train_mask;
  tr->n_train = n_train;
  tr->optimizer = d->optimizer;
  tr->shuffle = d->shuffle;
  tr->alpha_hist = d->alpha_hist;
  tr->history_swap = d->history_swap;
  tr->lr = d->lr;
  tr->beta1 = d->beta1;
  tr->beta2 = d->beta2;
  tr->eps = d->eps;
  tr->wd = d->weight_decay;
  tr->seed = d->seed;
  tr->ws = static_cast<char *>(d->workspace);
  tr->order.assign((size_t)x.K, 0);
  if (tr->optimizer == GNNTRAIN_ADAM && x.n_param_elems > 0) {
    const size_t bytes = sizeof(float) * (size_t)x.n_param_elems;
    if (launch_fill_zero(tr->at<char>(lay.m), bytes, nullptr) != 0 || launch_fill_zero(tr->at<char>(lay.v), bytes, nullptr) != 0 ||
        hipDeviceSynchronize() != hipSuccess)
      return bad(GNNSTAGE_EHIP, "clearing the optimiser state failed");
  }
  *out = holder.release();
  return GNNSTAGE_OK;
}
GNNSTAGE_GUARD_INT

extern "C" int gnntrain_destroy(gnntrain_t *tr) try {
  if (!tr) return GNNSTAGE_EINVAL;
  (void)hipDeviceSynchronize();
  delete tr;
  return GNNSTAGE_OK;
}
GNNSTAGE_GUARD_INT

extern "C" int gnntrain_last_order(const gnntrain_t *tr, int32_t *order) {
  if (!tr || !order) return GNNSTAGE_EINVAL;
  for (size_t i = 0; i < tr->order.size(); ++i) order[i] = tr->order[i];
  return GNNSTAGE_OK;
}

extern "C" int gnntrain_epoch(gnntrain_t *tr, int64_t epoch, float *loss, void *hip_stream) try {
  if (!tr) return GNNSTAGE_EINVAL;
  if (epoch < 0) return fail(tr, GNNSTAGE_EINVAL, "epoch must not be negative");
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const Dims &x = tr->x;
  const Layout &lay = tr->lay;
  const int cd = x.dtype;
  const int S = (int)tr->stages.size();
  gnntrain_chunk_order(tr->seed, epoch, x.K, tr->shuffle, tr->order.data());
  // dropout decisions of this epoch (stages without dropout ignore the seed): the epoch's SplitMix64 output, plus
  // the stage's index
  for (int s = 0; s < S; ++s)
    TRAIN_STAGE(tr, s, gnnstage_set_dropout_seed(tr->stages[(size_t)s], splitmix64(tr->seed + (uint64_t)(epoch + 1) * kGolden) + (uint64_t)s));

  for (const gnntrain_param &p : tr->params) TRAIN_HIP(tr, launch_fill_zero(p.grad, sizeof(float) * (size_t)p.count, stream));
  // the head's weights, staged like a layer's: transposed for the logits, plain for the input gradient
  TRAIN_HIP(tr, launch_stage_weights(tr->head_W, cd, x.d_top, x.C, tr->at<char>(lay.Wt), x.Kp, tr->at<char>(lay.Wn), x.Cp, stream));

  char *dlogits = tr->at<char>(lay.dlogits);
  float *row_loss = tr->at<float>(lay.row_loss);
  const float inv_n = (float)(1.0 / (double)tr->n_train);
  // ---- forward: every chunk through all stages, then through the head
  for (int pos = 0; pos < x.K; ++pos) {
    const int k = tr->order[(size_t)pos];
    for (int s = 0; s < S; ++s) TRAIN_STAGE(tr, s, stage_forward_chunk(tr->stages[(size_t)s], k, pos, stream));
    const int64_t row0 = tr->chunk_ptr[(size_t)k], M = tr->chunk_ptr[(size_t)k + 1] - row0;
    if (M == 0) continue;
    GemmNtArgs g{};
    g.A = static_cast<const char *>(tr->top) + (size_t)row0 * x.d_top * x.elt;
    g.a_dtype = cd;
    g.lda = x.d_top;
    g.Bt = tr->at<char>(lay.Wt);
    g.ldb = x.Kp;
    g.M = (int)M;
    g.N = x.C;
    g.K = x.d_top;
    g.Kp = x.Kp;
    g.epilogue = EPI_PLAIN;
    g.out = tr->at<float>(lay.logits);
    g.out_dtype = DT_F32;
    g.out_ld = x.Cp;
    TRAIN_HIP(tr, launch_gemm_nt(g, cd, stream));
    const int rc = gnntrain_softmax_xent(tr->at<float>(lay.logits), x.Cp, tr->head_b, tr->labels + row0, tr->mask ? tr->mask + row0 : nullptr,
                                         M, x.C, inv_n, dlogits + (size_t)row0 * x.Cp * x.elt, cd, x.Cp, row_loss + row0, stream);
    if (rc != GNNSTAGE_OK) return fail(tr, rc, "softmax cross-entropy launch failed");
  }
  // ---- backward: reverse order, head first, then the stages from the last to the first
  for (int pos = x.K - 1; pos >= 0; --pos) {
    const int k = tr->order[(size_t)pos];
    const int64_t row0 = tr->chunk_ptr[(size_t)k], M = tr->chunk_ptr[(size_t)k + 1] - row0;
    const char *dl = dlogits + (size_t)row0 * x.Cp * x.elt;
    const char *top_rows = static_cast<const char *>(tr->top) + (size_t)row0 * x.d_top * x.elt;
    char *dtop = tr->at<char>(lay.dtop);
    if (M > 0) {
      GemmTnArgs w{};
      w.A = top_rows;
      w.a_dtype = cd;
      w.lda = x.d_top;
      w.B = dl;
      w.ldb = x.Cp;
      w.M = (int)M;
      w.I = x.d_top;
      w.O = x.C;
      w.scale = 1.f;
      w.dW = tr->head_dW;
      w.partial = tr->at<float>(lay.gemm_partial);
      w.max_splits = kMaxSplits;
      if (cd == DT_BF16) {  // the bias gradient (column sums of the logit gradients) rides along
        w.dbias = tr->head_db;
        w.bias_partial = tr->at<float>(lay.bias_partial);
      }
      TRAIN_HIP(tr, launch_gemm_tn(w, cd, stream));
      if (cd != DT_BF16)
        TRAIN_HIP(tr, launch_colsum_add(dl, cd, x.Cp, (int)M, x.C, tr->at<float>(lay.bias_partial), kMaxSplits, tr->head_db, stream));
      GemmNtArgs g{};
      g.A = dl;
      g.a_dtype = cd;
      g.lda = x.Cp;
      g.Bt = tr->at<char>(lay.Wn);
      g.ldb = x.Cp;
      g.M = (int)M;
      g.N = x.d_top;
      g.K = x.C;
      g.Kp = x.Cp;
      g.epilogue = EPI_PLAIN;
      g.out = dtop;
      g.out_dtype = cd;
      g.out_ld = x.d_top;
      TRAIN_HIP(tr, launch_gemm_nt(g, cd, stream));
    }
    const char *gout = dtop;
    for (int s = S - 1; s >= 0; --s) {
      gnnstage_t *st = tr->stages[(size_t)s];
      TRAIN_STAGE(tr, s, stage_backward_chunk(st, k, gout, stream));
      if (s > 0) {
        const int d0 = (int)gnnstage_query(st, GNNSTAGE_Q_WIDTH, 0);
        gout = static_cast<const char *>(gnnstage_buffer(st, GNNSTAGE_B_GRAD_IN, 0)) + (size_t)row0 * d0 * x.elt;
      }
    }
  }
  // ---- the loss of this pass
  TRAIN_HIP(tr, launch_sum(row_loss, x.n, inv_n, tr->at<float>(lay.scratch), tr->at<float>(lay.loss), stream));
  // ---- weight update
  ++tr->step;
  for (size_t i = 0; i < tr->params.size(); ++i) {
    const gnntrain_param &p = tr->params[i];
    int rc;
    if (tr->optimizer == GNNTRAIN_ADAM)
      rc = gnntrain_adam_step(p.master, p.grad, tr->at<float>(lay.m) + tr->moment_off[i], tr->at<float>(lay.v) + tr->moment_off[i], p.compute,
                              p.compute_dtype, p.count, tr->lr, tr->beta1, tr->beta2, tr->eps, tr->wd, tr->step, stream);
    else
      rc = gnntrain_sgd_step(p.master, p.grad, p.compute, p.compute_dtype, p.count, tr->lr, tr->wd, stream);
    if (rc != GNNSTAGE_OK) return fail(tr, rc, "optimiser launch failed");
  }
  // ---- Section 3.4, second technique: the history of epoch alpha * floor((t - 1) / alpha)
  if ((epoch + 1) % tr->alpha_hist == 0)
    for (int s = 0; s < S; ++s) {
      if (tr->history_swap) TRAIN_STAGE(tr, s, gnnstage_update_history_swap(tr->stages[(size_t)s], stream));
      else TRAIN_STAGE(tr, s, update_history(tr->stages[(size_t)s], stream));
    }
  if (loss) {
    TRAIN_HIP(tr, hipMemcpyAsync(loss, tr->at<float>(lay.loss), sizeof(float), hipMemcpyDeviceToHost, stream));
    TRAIN_HIP(tr, hipStreamSynchronize(stream));
  }
  return GNNSTAGE_OK;
}
GNNSTAGE_GUARD_INT
