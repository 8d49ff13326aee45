// Small row-wise kernels of the epoch: ReLU' mask (Eq. 8) for callers that do not use the
// fused epilogues, and the softmax cross-entropy loss with its gradient.
#include "common.h"

#include <algorithm>
#include <cmath>
#include <mutex>

namespace mggcn {
namespace {

constexpr int kThreads = 256;

// Loss partials of mggcn_softmax_ce_static: one per workgroup of the loss kernel, whose grid never
// exceeds this many workgroups.  The array lives in every GPU's memory from the moment the library's
// code is loaded there until the process ends (16 KiB per GPU).  In host code the name is only a
// handle for hipGetSymbolAddress; kernels are given the address that call returns.
constexpr int kStaticLossPartials = 4096;
static __device__ __align__(256) float scratch[kStaticLossPartials];

__global__ __launch_bounds__(kThreads) void relu_bwd_kernel(int64_t rows, int cols,
                                                             const float* __restrict__ act,
                                                             int64_t lda, float* __restrict__ G,
                                                             int64_t ldg) {
  const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= rows * cols) return;
  const int64_t i = idx / cols;
  const int f = (int)(idx % cols);
  if (!(act[i * lda + f] > 0.f)) G[i * ldg + f] = 0.f;
}

// T lanes (power of two, <= 64) per row; 64/T rows per wavefront per step; a fixed grid whose
// wavefronts stride over the rows, so the number of loss partials stays small and every partial
// is summed in a fixed order.
__global__ __launch_bounds__(kThreads) void softmax_ce_kernel(int64_t n, int C, int T,
                                                               const float* Z, int64_t ldz,
                                                               const int32_t* __restrict__ labels,
                                                               float* dZ, int64_t ldd,
                                                               float inv_n,
                                                               float* __restrict__ block_loss) {
  __shared__ float wave_loss[kThreads / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int rows_per_wave = 64 / T;
  const int tl = lane % T;
  const int64_t wave_gid = (int64_t)blockIdx.x * (kThreads / 64) + wave;
  const int64_t n_waves = (int64_t)gridDim.x * (kThreads / 64);
  float loss_acc = 0.f;
  for (int64_t base = wave_gid * rows_per_wave; base < n; base += n_waves * rows_per_wave) {
    const int64_t row = base + lane / T;
    const bool live = row < n;
    const float* z = Z + (live ? row : 0) * ldz;
    float mx = -INFINITY;
    if (live)
      for (int c = tl; c < C; c += T) mx = fmaxf(mx, z[c]);
    for (int d = 1; d < T; d <<= 1) mx = fmaxf(mx, __shfl_xor(mx, d));
    float s = 0.f;
    if (live)
      for (int c = tl; c < C; c += T) s += expf(z[c] - mx);
    for (int d = 1; d < T; d <<= 1) s += __shfl_xor(s, d);
    float lse = 0.f, others = 0.f;
    int y = -1;
    if (live) {
      lse = mx + logf(s);
      y = labels[row];
      for (int c = tl; c < C; c += T)
        if (c != y) others += expf(z[c] - lse);
    }
    // softmax[y] - 1 = -(sum of the other classes): free of cancellation when softmax[y] -> 1
    for (int d = 1; d < T; d <<= 1) others += __shfl_xor(others, d);
    if (live) {
      float* g = dZ + row * ldd;  // may be the same memory as z: each lane reads an element
      for (int c = tl; c < C; c += T) {  // before it overwrites that same element
        const float zc = z[c];
        if (c == y) loss_acc += lse - zc;
        g[c] = (c == y ? -others : expf(zc - lse)) * inv_n;
      }
    }
  }
  // fixed-order reduction: lanes by xor tree, wavefronts in index order
  for (int d = 1; d < 64; d <<= 1) loss_acc += __shfl_xor(loss_acc, d);
  if (lane == 0) wave_loss[wave] = loss_acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = 0.f;
    for (int w = 0; w < kThreads / 64; ++w) t += wave_loss[w];
    block_loss[blockIdx.x] = t;
  }
}

// The same loss for rows of up to 64 * 8 classes, with the row held in registers: T lanes share a
// row, each holding E elements (column tl + T*e), so logits are read once and written once and
// one exponential is taken per element (softmax = exp(z - max) / sum, the label's entry again as
// minus the sum of the others).  Same grid and same fixed-order loss partials as the general
// kernel above.
template <int E>
__global__ __launch_bounds__(kThreads) void softmax_ce_rows(int64_t n, int C, int T, const float* Z, int64_t ldz,
                                                             const int32_t* __restrict__ labels, float* dZ,
                                                             int64_t ldd, float inv_n,
                                                             float* __restrict__ block_loss) {
  __shared__ float wave_loss[kThreads / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int rows_per_wave = 64 / T;
  const int tl = lane % T;
  const int64_t wave_gid = (int64_t)blockIdx.x * (kThreads / 64) + wave;
  const int64_t n_waves = (int64_t)gridDim.x * (kThreads / 64);
  float loss_acc = 0.f;
  for (int64_t base = wave_gid * rows_per_wave; base < n; base += n_waves * rows_per_wave) {
    const int64_t row = base + lane / T;
    const bool live = row < n;
    const float* z = Z + (live ? row : 0) * ldz;
    float v[E];
    float mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const int c = tl + T * e;
      v[e] = (live && c < C) ? z[c] : -INFINITY;
      mx = fmaxf(mx, v[e]);
    }
    for (int d = 1; d < T; d <<= 1) mx = fmaxf(mx, __shfl_xor(mx, d));
    const int y = live ? labels[row] : -1;
    float s = 0.f, others = 0.f, zy = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const int c = tl + T * e;
      const float ex = (live && c < C) ? expf(v[e] - mx) : 0.f;
      s += ex;
      if (c == y) zy = v[e]; else others += ex;
      v[e] = ex;
    }
    for (int d = 1; d < T; d <<= 1) {
      s += __shfl_xor(s, d);
      others += __shfl_xor(others, d);
      zy += __shfl_xor(zy, d);  // one lane of the team holds the label's logit, the rest 0
    }
    if (live) {
      const float inv = 1.f / s;
      if (tl == 0) loss_acc += mx + logf(s) - zy;
      float* g = dZ + row * ldd;  // may be the same memory as z: the row is already in registers
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const int c = tl + T * e;
        if (c < C) g[c] = (c == y ? -others : v[e]) * inv * inv_n;
      }
    }
  }
  for (int d = 1; d < 64; d <<= 1) loss_acc += __shfl_xor(loss_acc, d);
  if (lane == 0) wave_loss[wave] = loss_acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = 0.f;
    for (int w = 0; w < kThreads / 64; ++w) t += wave_loss[w];
    block_loss[blockIdx.x] = t;
  }
}

__global__ __launch_bounds__(kThreads) void loss_finish(int64_t nblocks,
                                                         const float* __restrict__ block_loss,
                                                         double inv_n, float* __restrict__ loss) {
  __shared__ double part[kThreads];
  double s = 0.0;
  for (int64_t b = threadIdx.x; b < nblocks; b += kThreads) s += (double)block_loss[b];
  part[threadIdx.x] = s;
  __syncthreads();
  for (int d = kThreads / 2; d > 0; d >>= 1) {
    if ((int)threadIdx.x < d) part[threadIdx.x] += part[threadIdx.x + d];
    __syncthreads();
  }
  if (threadIdx.x == 0) *loss = (float)(part[0] * inv_n);
}

__global__ __launch_bounds__(kThreads) void adam_kernel(int64_t count, float* __restrict__ W,
                                                         const float* __restrict__ G, float* __restrict__ m,
                                                         float* __restrict__ v, float lr, float b1, float b2,
                                                         float eps, float inv_c1, float inv_c2) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= count) return;
  const float g = G[i];
  const float mi = b1 * m[i] + (1.f - b1) * g;
  const float vi = b2 * v[i] + (1.f - b2) * g * g;
  m[i] = mi;
  v[i] = vi;
  W[i] -= lr * (mi * inv_c1) / (sqrtf(vi * inv_c2) + eps);
}

// Lanes per row: about four elements per lane (so that several narrow rows share a wavefront and a
// lane still reads 16-lane-wide contiguous pieces), at least 4, at most 64.
int team_lanes(int C) {
  int t = 4;
  while (t * 4 < C && t < 64) t <<= 1;
  return t;
}

int64_t loss_blocks(int64_t n, int C) {
  const int rows_per_block = (kThreads / 64) * (64 / team_lanes(C));
  return std::min<int64_t>(ceil_div(n, rows_per_block), kStaticLossPartials);
}

// Address of `scratch` on the current device, looked up once per device (each GPU holds its own
// copy of the array at its own address).
int static_scratch(float** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static float* ptrs[kMaxDevices] = {};
  int dev = -1;
  MGGCN_HIP(hipGetDevice(&dev));
  MGGCN_REQUIRE(dev >= 0 && dev < kMaxDevices, MGGCN_E_UNSUPPORTED, "device index %d outside [0, %d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(mu);
  if (ptrs[dev] == nullptr) {
    void* p = nullptr;
    MGGCN_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    MGGCN_REQUIRE(p != nullptr, MGGCN_E_HIP, "hipGetSymbolAddress returned a null address");
    ptrs[dev] = static_cast<float*>(p);
  }
  *out = ptrs[dev];
  return MGGCN_OK;
}

int softmax_ce_check(int64_t n, int32_t C, const float* logits, int64_t ld, const int32_t* labels,
                     const float* loss_dev, const float* dlogits, int64_t ldd) {
  MGGCN_REQUIRE(n > 0 && C > 0, MGGCN_E_INVALID_ARG, "need n > 0 and C > 0 (n=%lld, C=%d)", (long long)n, C);
  MGGCN_REQUIRE(ld >= C && ldd >= C, MGGCN_E_INVALID_ARG, "leading dimension < C");
  MGGCN_REQUIRE(logits && labels && loss_dev && dlogits, MGGCN_E_INVALID_ARG, "NULL argument");
  return MGGCN_OK;
}

// The two launches of the loss: per-workgroup partials into block_loss (every entry below `blocks`
// is written, none is read before), then their sum in a fixed order.
int softmax_ce_run(int64_t n, int32_t C, const float* logits, int64_t ld, const int32_t* labels, float* loss_dev,
                   float* dlogits, int64_t ldd, float* block_loss, hipStream_t s) {
  const int64_t blocks = loss_blocks(n, C);
  const int T = team_lanes(C);
  const float inv_n = (float)(1.0 / (double)n);
  switch ((int)ceil_div(C, T)) {  // elements per lane
    case 1: softmax_ce_rows<1><<<(unsigned)blocks, kThreads, 0, s>>>(n, C, T, logits, ld, labels, dlogits, ldd, inv_n, block_loss); break;
    case 2: softmax_ce_rows<2><<<(unsigned)blocks, kThreads, 0, s>>>(n, C, T, logits, ld, labels, dlogits, ldd, inv_n, block_loss); break;
    case 3: softmax_ce_rows<3><<<(unsigned)blocks, kThreads, 0, s>>>(n, C, T, logits, ld, labels, dlogits, ldd, inv_n, block_loss); break;
    case 4: softmax_ce_rows<4><<<(unsigned)blocks, kThreads, 0, s>>>(n, C, T, logits, ld, labels, dlogits, ldd, inv_n, block_loss); break;
    case 5: case 6: case 7: case 8:
      softmax_ce_rows<8><<<(unsigned)blocks, kThreads, 0, s>>>(n, C, T, logits, ld, labels, dlogits, ldd, inv_n, block_loss); break;
    default:  // more than 512 classes: the general kernel walks the row in passes
      softmax_ce_kernel<<<(unsigned)blocks, kThreads, 0, s>>>(n, C, T, logits, ld, labels, dlogits, ldd, inv_n, block_loss);
  }
  MGGCN_LAUNCH_CHECK();
  loss_finish<<<1, kThreads, 0, s>>>(blocks, block_loss, 1.0 / (double)n, loss_dev);
  MGGCN_LAUNCH_CHECK();
  return MGGCN_OK;
}

}  // namespace
}  // namespace mggcn

using namespace mggcn;

extern "C" {

int mggcn_relu_bwd(int64_t rows, int32_t cols, const float* act, int64_t lda, float* G, int64_t ldg,
                   void* stream) {
  MGGCN_REQUIRE(rows >= 0 && cols >= 0, MGGCN_E_INVALID_ARG, "negative size %lld x %d", (long long)rows, cols);
  MGGCN_REQUIRE(lda >= cols && ldg >= cols, MGGCN_E_INVALID_ARG, "leading dimension < cols");
  if (rows == 0 || cols == 0) return MGGCN_OK;
  MGGCN_REQUIRE(act && G, MGGCN_E_INVALID_ARG, "act / G is NULL");
  const int64_t blocks = ceil_div(rows * cols, kThreads);
  MGGCN_REQUIRE(blocks < ((int64_t)1 << 31), MGGCN_E_OVERFLOW, "matrix too large for one launch");
  relu_bwd_kernel<<<(unsigned)blocks, kThreads, 0, as_stream(stream)>>>(rows, cols, act, lda, G, ldg);
  MGGCN_LAUNCH_CHECK();
  return MGGCN_OK;
}

int mggcn_adam_step(int64_t count, float* W, const float* G, float* m, float* v, int32_t step, float lr,
                    float beta1, float beta2, float eps, void* stream) {
  MGGCN_REQUIRE(count >= 0, MGGCN_E_INVALID_ARG, "negative count %lld", (long long)count);
  MGGCN_REQUIRE(step >= 1, MGGCN_E_INVALID_ARG, "step %d must start at 1", step);
  MGGCN_REQUIRE(beta1 >= 0.f && beta1 < 1.f && beta2 >= 0.f && beta2 < 1.f, MGGCN_E_INVALID_ARG,
                "beta1 / beta2 must lie in [0, 1)");
  if (count == 0) return MGGCN_OK;
  MGGCN_REQUIRE(W && G && m && v, MGGCN_E_INVALID_ARG, "NULL argument");
  const int64_t blocks = ceil_div(count, kThreads);
  MGGCN_REQUIRE(blocks < ((int64_t)1 << 31), MGGCN_E_OVERFLOW, "too many parameters for one launch");
  // bias corrections evaluated once on the host in double
  const double c1 = 1.0 - pow((double)beta1, (double)step), c2 = 1.0 - pow((double)beta2, (double)step);
  adam_kernel<<<(unsigned)blocks, kThreads, 0, as_stream(stream)>>>(count, W, G, m, v, lr, beta1, beta2, eps,
                                                                   (float)(1.0 / c1), (float)(1.0 / c2));
  MGGCN_LAUNCH_CHECK();
  return MGGCN_OK;
}

size_t mggcn_softmax_ce_workspace_bytes(int64_t n) {
  if (n <= 0) return 0;
  // worst case one row per wavefront
  return align_up((size_t)ceil_div(n, kThreads / 64) * sizeof(float), kWsAlign);
}

int mggcn_softmax_ce(int64_t n, int32_t C, const float* logits, int64_t ld, const int32_t* labels,
                     float* loss_dev, float* dlogits, int64_t ldd, void* ws, size_t ws_bytes,
                     void* stream) {
  const int rc = softmax_ce_check(n, C, logits, ld, labels, loss_dev, dlogits, ldd);
  if (rc) return rc;
  MGGCN_REQUIRE(ws && aligned(ws, kWsAlign), MGGCN_E_WORKSPACE, "workspace is NULL or not 256-byte aligned");
  MGGCN_REQUIRE(ws_bytes >= mggcn_softmax_ce_workspace_bytes(n), MGGCN_E_WORKSPACE,
                "workspace too small: %zu bytes given, %zu needed", ws_bytes,
                mggcn_softmax_ce_workspace_bytes(n));
  return softmax_ce_run(n, C, logits, ld, labels, loss_dev, dlogits, ldd, static_cast<float*>(ws), as_stream(stream));
}

int mggcn_softmax_ce_static(int64_t n, int32_t C, const float* logits, int64_t ld, const int32_t* labels,
                            float* loss_dev, float* dlogits, int64_t ldd, void* stream) {
  int rc = softmax_ce_check(n, C, logits, ld, labels, loss_dev, dlogits, ldd);
  if (rc) return rc;
  MGGCN_REQUIRE(n <= MGGCN_SOFTMAX_CE_STATIC_MAX_ROWS, MGGCN_E_UNSUPPORTED,
                "n = %lld exceeds the %lld rows mggcn_softmax_ce_static takes; use mggcn_softmax_ce with a workspace",
                (long long)n, (long long)MGGCN_SOFTMAX_CE_STATIC_MAX_ROWS);
  MGGCN_REQUIRE(loss_blocks(n, C) <= kStaticLossPartials, MGGCN_E_UNSUPPORTED,
                "the loss needs %lld partial sums, the built-in buffer holds %d", (long long)loss_blocks(n, C),
                kStaticLossPartials);
  float* partials = nullptr;
  rc = static_scratch(&partials);
  if (rc) return rc;
  return softmax_ce_run(n, C, logits, ld, labels, loss_dev, dlogits, ldd, partials, as_stream(stream));
}

}  // extern "C"
