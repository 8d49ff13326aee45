// Error reporting and the prefix sums (int32 counts to int32 or int64 offsets) used by the setup kernels.
#include "common.h"

#include <cstring>

namespace mggcn {

char* error_buffer() {
  static thread_local char buf[512] = {0};
  return buf;
}

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(error_buffer(), 512, fmt, ap);
  va_end(ap);
  return code;
}

namespace {

constexpr int kScanThreads = 256;
constexpr int kScanItems = 4;
constexpr int kScanTile = kScanThreads * kScanItems;

template <typename T>
__device__ inline T wave_inclusive_scan(T v, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    T t = __shfl_up(v, d);
    if (lane >= d) v += t;
  }
  return v;
}

// Inclusive scan of one value per thread over a 256-thread block; returns the exclusive
// prefix of this thread and the block total through *total.
template <typename T>
__device__ inline T block_exclusive_scan(T v, T* total) {
  __shared__ T wave_sum[kScanThreads / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const T inc = wave_inclusive_scan<T>(v, lane);
  if (lane == 63) wave_sum[wave] = inc;
  __syncthreads();
  T off = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kScanThreads / 64; ++w) {
    const T s = wave_sum[w];
    if (w < wave) off += s;
    tot += s;
  }
  __syncthreads();
  *total = tot;
  return off + inc - v;
}

template <typename IN, typename T>
__global__ __launch_bounds__(kScanThreads) void scan_tile_sums(const IN* __restrict__ in, int64_t n,
                                                                T* __restrict__ sums) {
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
  T v = 0;
#pragma unroll
  for (int i = 0; i < kScanItems; ++i)
    if (base + i < n) v += (T)in[base + i];
  T total;
  block_exclusive_scan<T>(v, &total);
  if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

// offsets == nullptr: single tile.  Writes out[i] for i < n and out[n] (last tile).
template <typename IN, typename T>
__global__ __launch_bounds__(kScanThreads) void scan_tiles(const IN* __restrict__ in, int64_t n,
                                                           const T* __restrict__ offsets, T* __restrict__ out) {
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
  T item[kScanItems];
  T v = 0;
#pragma unroll
  for (int i = 0; i < kScanItems; ++i) {
    item[i] = (base + i < n) ? (T)in[base + i] : (T)0;
    v += item[i];
  }
  T total;
  T run = block_exclusive_scan<T>(v, &total) + (offsets ? offsets[blockIdx.x] : (T)0);
#pragma unroll
  for (int i = 0; i < kScanItems; ++i) {
    if (base + i < n) out[base + i] = run;
    run += item[i];
    if (base + i == n - 1) out[n] = run;
  }
  if (n == 0 && blockIdx.x == 0 && threadIdx.x == 0) out[0] = 0;
}

template <typename IN, typename T>
int exclusive_scan_impl(const IN* counts, int64_t n, T* out, T* tmp, hipStream_t s) {
  if (n <= kScanTile) {
    scan_tiles<IN, T><<<1, kScanThreads, 0, s>>>(counts, n, nullptr, out);
    MGGCN_LAUNCH_CHECK();
    return MGGCN_OK;
  }
  const int64_t nb = ceil_div(n, kScanTile);
  T* sums = tmp;
  T* offs = tmp + align_up((size_t)nb, 64);
  T* rest = offs + align_up((size_t)nb + 1, 64);
  scan_tile_sums<IN, T><<<(unsigned)nb, kScanThreads, 0, s>>>(counts, n, sums);
  MGGCN_LAUNCH_CHECK();
  int rc = exclusive_scan_impl<T, T>(sums, nb, offs, rest, s);
  if (rc) return rc;
  scan_tiles<IN, T><<<(unsigned)nb, kScanThreads, 0, s>>>(counts, n, offs, out);
  MGGCN_LAUNCH_CHECK();
  return MGGCN_OK;
}

}  // namespace

size_t scan_tmp_ints(int64_t n) {
  size_t total = 0;
  while (n > kScanTile) {
    const int64_t nb = ceil_div(n, kScanTile);
    total += align_up((size_t)nb, 64) + align_up((size_t)nb + 1, 64);
    n = nb;
  }
  return total + 64;
}

int exclusive_scan_i32(const int32_t* counts, int64_t n, int32_t* out, int32_t* tmp, hipStream_t s) {
  return exclusive_scan_impl<int32_t, int32_t>(counts, n, out, tmp, s);
}

int exclusive_scan_i64(const int32_t* counts, int64_t n, int64_t* out, int64_t* tmp, hipStream_t s) {
  return exclusive_scan_impl<int32_t, int64_t>(counts, n, out, tmp, s);
}

}  // namespace mggcn

extern "C" {

const char* mggcn_last_error(void) { return mggcn::error_buffer(); }

int mggcn_version(void) { return 100; }

}  // extern "C"
