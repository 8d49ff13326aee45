// Error reporting and the int32 prefix-sum used by the setup kernels.
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

__device__ inline int wave_inclusive_scan(int v, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    int t = __shfl_up(v, d);
    if (lane >= d) v += t;
  }
  return v;
}

// Inclusive scan of one value per thread over a 256-thread block; returns the exclusive
// prefix of this thread and the block total through *total.
__device__ inline int block_exclusive_scan(int v, int* total) {
  __shared__ int wave_sum[kScanThreads / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int inc = wave_inclusive_scan(v, lane);
  if (lane == 63) wave_sum[wave] = inc;
  __syncthreads();
  int off = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kScanThreads / 64; ++w) {
    const int s = wave_sum[w];
    if (w < wave) off += s;
    tot += s;
  }
  __syncthreads();
  *total = tot;
  return off + inc - v;
}

__global__ __launch_bounds__(kScanThreads) void scan_tile_sums(const int32_t* __restrict__ in,
                                                                int64_t n,
                                                                int32_t* __restrict__ sums) {
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
  int v = 0;
#pragma unroll
  for (int i = 0; i < kScanItems; ++i)
    if (base + i < n) v += in[base + i];
  int total;
  block_exclusive_scan(v, &total);
  if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

// offsets == nullptr: single tile.  Writes out[i] for i < n and out[n] (last tile).
__global__ __launch_bounds__(kScanThreads) void scan_tiles(const int32_t* __restrict__ in,
                                                           int64_t n,
                                                           const int32_t* __restrict__ offsets,
                                                           int32_t* __restrict__ out) {
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
  int item[kScanItems];
  int v = 0;
#pragma unroll
  for (int i = 0; i < kScanItems; ++i) {
    item[i] = (base + i < n) ? in[base + i] : 0;
    v += item[i];
  }
  int total;
  int run = block_exclusive_scan(v, &total) + (offsets ? offsets[blockIdx.x] : 0);
#pragma unroll
  for (int i = 0; i < kScanItems; ++i) {
    if (base + i < n) out[base + i] = run;
    run += item[i];
    if (base + i == n - 1) out[n] = run;
  }
  if (n == 0 && blockIdx.x == 0 && threadIdx.x == 0) out[0] = 0;
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
  if (n <= kScanTile) {
    scan_tiles<<<1, kScanThreads, 0, s>>>(counts, n, nullptr, out);
    MGGCN_LAUNCH_CHECK();
    return MGGCN_OK;
  }
  const int64_t nb = ceil_div(n, kScanTile);
  int32_t* sums = tmp;
  int32_t* offs = tmp + align_up((size_t)nb, 64);
  int32_t* rest = offs + align_up((size_t)nb + 1, 64);
  scan_tile_sums<<<(unsigned)nb, kScanThreads, 0, s>>>(counts, n, sums);
  MGGCN_LAUNCH_CHECK();
  int rc = exclusive_scan_i32(sums, nb, offs, rest, s);
  if (rc) return rc;
  scan_tiles<<<(unsigned)nb, kScanThreads, 0, s>>>(counts, n, offs, out);
  MGGCN_LAUNCH_CHECK();
  return MGGCN_OK;
}

}  // namespace mggcn

extern "C" {

const char* mggcn_last_error(void) { return mggcn::error_buffer(); }

int mggcn_version(void) { return 100; }

}  // extern "C"
