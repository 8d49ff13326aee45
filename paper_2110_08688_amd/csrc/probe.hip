// Memory-system probes: what this GPU delivers for the two access patterns the SpMM consists of,
// measured by the benchmark in the same run as the SpMM itself and quoted next to the datasheet
// bandwidth.  Not part of the training path.
//
//   read / write stream : every workgroup reads (fills) a contiguous share of a buffer with 16-byte
//                 loads (stores) -- the
//                 pattern of the column-index / value streams and of any dense pass over a matrix.
//   row gather  : rows of a dense matrix are fetched in the order an index list gives, LPR lanes x
//                 16 bytes per row, eight rows in flight per lane -- the pattern of the SpMM's
//                 gathers (Eq. 6, 9) with the arithmetic, the value stream and the output removed.
//
// Both keep a running sum per lane and store one number per workgroup, so the loads cannot be
// dropped and the stores are negligible.  A third probe issues nothing but the fp32 matrix
// instruction of the GeMM (Eq. 5, 10, 11) on register operands.
#include "common.h"

#include <algorithm>

namespace mggcn {
namespace {

constexpr int kThreads = 256;
constexpr int kProbeBlocks = 4096;  // sink entries a probe writes at most

typedef float vec4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kThreads) void probe_read_kernel(const vec4* __restrict__ buf, int64_t n_vec,
                                                               float* __restrict__ sink) {
  // a workgroup walks its own contiguous share; consecutive lanes read consecutive 16 bytes
  const int64_t per_block = (n_vec + gridDim.x - 1) / gridDim.x;
  const int64_t begin = (int64_t)blockIdx.x * per_block;
  const int64_t end = min(n_vec, begin + per_block);
  float s = 0.f;
  int64_t i = begin + threadIdx.x;
  for (; i + 3 * kThreads < end; i += 4 * kThreads) {
    const vec4 a = __builtin_nontemporal_load(buf + i);
    const vec4 b = __builtin_nontemporal_load(buf + i + kThreads);
    const vec4 c = __builtin_nontemporal_load(buf + i + 2 * kThreads);
    const vec4 d = __builtin_nontemporal_load(buf + i + 3 * kThreads);
    s += (a.x + a.y + a.z + a.w) + (b.x + b.y + b.z + b.w) + (c.x + c.y + c.z + c.w) + (d.x + d.y + d.z + d.w);
  }
  for (; i < end; i += kThreads) {
    const vec4 a = __builtin_nontemporal_load(buf + i);
    s += a.x + a.y + a.z + a.w;
  }
  for (int d = 1; d < 64; d <<= 1) s += __shfl_xor(s, d);
  __shared__ float part[kThreads / 64];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) sink[blockIdx.x] = part[0] + part[1] + part[2] + part[3];
}

// write stream: every workgroup fills a contiguous share with 16-byte stores
__global__ __launch_bounds__(kThreads) void probe_write_kernel(vec4* __restrict__ buf, int64_t n_vec, float value) {
  const int64_t per_block = (n_vec + gridDim.x - 1) / gridDim.x;
  const int64_t begin = (int64_t)blockIdx.x * per_block;
  const int64_t end = min(n_vec, begin + per_block);
  const vec4 v = {value, value, value, value};
  for (int64_t i = begin + threadIdx.x; i < end; i += kThreads) buf[i] = v;
}

template <int LPR>
__global__ __launch_bounds__(kThreads) void probe_gather_kernel(const char* __restrict__ X, uint32_t last_row,
                                                                 uint32_t row_stride, const int32_t* __restrict__ idx,
                                                                 int64_t n_idx, float* __restrict__ sink) {
  constexpr int TPB = kThreads / LPR;  // rows a workgroup fetches at a time, one per team of LPR lanes
  constexpr int U = 8;                 // rows in flight per lane
  const int team = threadIdx.x / LPR, fl = threadIdx.x % LPR;
  const int64_t n_teams = (int64_t)gridDim.x * TPB;
  const char* __restrict__ xl = X + fl * 16;
  float s = 0.f;
  int64_t k = (int64_t)blockIdx.x * TPB + team;
  for (; k + (U - 1) * n_teams < n_idx; k += U * n_teams) {
    uint32_t r[U];
    float4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) r[u] = min((uint32_t)idx[k + u * n_teams], last_row);  // never outside X
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = *reinterpret_cast<const float4*>(xl + (uint64_t)r[u] * row_stride);
#pragma unroll
    for (int u = 0; u < U; ++u) s += (v[u].x + v[u].y) + (v[u].z + v[u].w);
  }
  for (; k < n_idx; k += n_teams) {
    const float4 a = *reinterpret_cast<const float4*>(xl + (uint64_t)min((uint32_t)idx[k], last_row) * row_stride);
    s += a.x + a.y + a.z + a.w;
  }
  for (int d = 1; d < 64; d <<= 1) s += __shfl_xor(s, d);
  __shared__ float part[kThreads / 64];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) sink[blockIdx.x] = part[0] + part[1] + part[2] + part[3];
}

// Sustained issue rate of the fp32 matrix instruction the GeMM is built on, operands in registers,
// nothing else going on: 32 independent-enough instructions (four accumulators) per loop trip.
typedef float probe_acc __attribute__((ext_vector_type(16)));
constexpr int kMfmaProbeBlocks = 512;  // two workgroups per CU: two wavefronts per SIMD
__global__ __launch_bounds__(kThreads) void probe_mfma_kernel(int iters, float* __restrict__ sink) {
  probe_acc acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  const float a = 1.f + (float)(threadIdx.x & 7) * 0.125f, b = 1.f - (float)(threadIdx.x & 3) * 0.25f;
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[j][r];
  for (int d = 1; d < 64; d <<= 1) s += __shfl_xor(s, d);
  __shared__ float part[kThreads / 64];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) sink[blockIdx.x] = part[0] + part[1] + part[2] + part[3];
}

}  // namespace
}  // namespace mggcn

using namespace mggcn;

extern "C" {

int32_t mggcn_probe_sink_floats(void) { return kProbeBlocks; }

int mggcn_probe_read(const void* buf, int64_t bytes, float* sink, void* stream) {
  MGGCN_REQUIRE(bytes >= 0 && bytes % 16 == 0, MGGCN_E_INVALID_ARG, "bytes = %lld must be a non-negative multiple of 16",
                (long long)bytes);
  if (bytes == 0) return MGGCN_OK;
  MGGCN_REQUIRE(buf && sink && aligned(buf, 16), MGGCN_E_INVALID_ARG, "buf / sink is NULL or buf is not 16-byte aligned");
  const int64_t n_vec = bytes / 16;
  const int blocks = (int)std::min<int64_t>(kProbeBlocks, ceil_div(n_vec, kThreads));
  probe_read_kernel<<<blocks, kThreads, 0, as_stream(stream)>>>(static_cast<const vec4*>(buf), n_vec, sink);
  MGGCN_LAUNCH_CHECK();
  return MGGCN_OK;
}

int mggcn_probe_write(void* buf, int64_t bytes, float value, void* stream) {
  MGGCN_REQUIRE(bytes >= 0 && bytes % 16 == 0, MGGCN_E_INVALID_ARG, "bytes = %lld must be a non-negative multiple of 16",
                (long long)bytes);
  if (bytes == 0) return MGGCN_OK;
  MGGCN_REQUIRE(buf && aligned(buf, 16), MGGCN_E_INVALID_ARG, "buf is NULL or not 16-byte aligned");
  const int64_t n_vec = bytes / 16;
  const int blocks = (int)std::min<int64_t>(kProbeBlocks, ceil_div(n_vec, kThreads));
  probe_write_kernel<<<blocks, kThreads, 0, as_stream(stream)>>>(static_cast<vec4*>(buf), n_vec, value);
  MGGCN_LAUNCH_CHECK();
  return MGGCN_OK;
}

int64_t mggcn_probe_mfma(int32_t iters, float* sink, void* stream) {
  if (iters < 1 || iters > (1 << 24) || !sink) {
    fail(MGGCN_E_INVALID_ARG, "iters %d outside [1, 2^24] or sink is NULL", iters);
    return MGGCN_E_INVALID_ARG;
  }
  probe_mfma_kernel<<<kMfmaProbeBlocks, kThreads, 0, as_stream(stream)>>>(iters, sink);
  if (hipGetLastError() != hipSuccess) {
    fail(MGGCN_E_HIP, "probe launch failed");
    return MGGCN_E_HIP;
  }
  // workgroups x wavefronts x trips x instructions x (2 x 32 x 32 x 2 flop)
  return (int64_t)kMfmaProbeBlocks * (kThreads / 64) * (int64_t)iters * 32 * 4096;
}

int mggcn_probe_gather(const void* X, int64_t n_rows, int32_t row_bytes, int64_t row_stride, const int32_t* idx,
                       int64_t n_idx, float* sink, void* stream) {
  MGGCN_REQUIRE(n_rows >= 1 && n_idx >= 0, MGGCN_E_INVALID_ARG, "need n_rows >= 1 and n_idx >= 0");
  MGGCN_REQUIRE(row_bytes == 64 || row_bytes == 128 || row_bytes == 256 || row_bytes == 512 || row_bytes == 1024,
                MGGCN_E_INVALID_ARG, "row_bytes = %d must be 64, 128, 256, 512 or 1024", row_bytes);
  MGGCN_REQUIRE(row_stride >= row_bytes && row_stride % 16 == 0 && row_stride < ((int64_t)1 << 32), MGGCN_E_INVALID_ARG,
                "row_stride %lld must be a multiple of 16 in [row_bytes, 2^32)", (long long)row_stride);
  MGGCN_REQUIRE(n_rows < ((int64_t)1 << 31), MGGCN_E_OVERFLOW, "n_rows must fit 31 bits");
  if (n_idx == 0) return MGGCN_OK;
  MGGCN_REQUIRE(X && idx && sink && aligned(X, 16), MGGCN_E_INVALID_ARG, "X / idx / sink is NULL or X is not 16-byte aligned");
  const int lpr = row_bytes / 16;
  const int blocks = (int)std::min<int64_t>(kProbeBlocks, ceil_div(n_idx, kThreads / lpr));
  const char* x = static_cast<const char*>(X);
  hipStream_t s = as_stream(stream);
  switch (lpr) {
    case 4: probe_gather_kernel<4><<<blocks, kThreads, 0, s>>>(x, (uint32_t)(n_rows - 1), (uint32_t)row_stride, idx, n_idx, sink); break;
    case 8: probe_gather_kernel<8><<<blocks, kThreads, 0, s>>>(x, (uint32_t)(n_rows - 1), (uint32_t)row_stride, idx, n_idx, sink); break;
    case 16: probe_gather_kernel<16><<<blocks, kThreads, 0, s>>>(x, (uint32_t)(n_rows - 1), (uint32_t)row_stride, idx, n_idx, sink); break;
    case 32: probe_gather_kernel<32><<<blocks, kThreads, 0, s>>>(x, (uint32_t)(n_rows - 1), (uint32_t)row_stride, idx, n_idx, sink); break;
    default: probe_gather_kernel<64><<<blocks, kThreads, 0, s>>>(x, (uint32_t)(n_rows - 1), (uint32_t)row_stride, idx, n_idx, sink); break;
  }
  MGGCN_LAUNCH_CHECK();
  return MGGCN_OK;
}

}  // extern "C"
