// Stable least-significant-digit radix sort of (key, value) pairs of 32 unsigned bits, eight key bits
// per pass.  Setup code: the explicit transpose of A^ (entries ordered by column, rows ascending
// inside a column) and the longest-first order of the SpMM's row segments are both stable sorts of
// small integer keys.  Stability makes the result unique, so it is reproducible bit for bit.
//
// One pass over n pairs, tiles of 2048 pairs per workgroup:
//   radix_hist     per-tile count of each of the 256 digit values (LDS integer atomics), written
//                  digit-major so that one prefix sum over the whole table ...
//   (scan)         ... gives, for every (digit, tile), where that tile's first pair with that digit goes;
//   radix_scatter  every wavefront owns 512 consecutive pairs of the tile and walks them 64 at a time in
//                  order: lanes holding the same digit find each other with eight ballots, a lane's place
//                  among them is the number of such lanes below it, and a per-wavefront running count per
//                  digit carries the order from one step to the next.
#include "common.h"

namespace mggcn {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kItems = 8;                      // pairs per thread
constexpr int kTile = kThreads * kItems;       // pairs per workgroup
constexpr int kWaveTile = kTile / kWaves;      // consecutive pairs per wavefront
constexpr int kDigits = 256;

__global__ __launch_bounds__(kThreads) void radix_hist(const uint32_t* __restrict__ keys, int64_t n, int shift,
                                                        int32_t* __restrict__ hist, int64_t n_tiles) {
  __shared__ uint32_t h[kDigits];
  h[threadIdx.x] = 0u;
  __syncthreads();
  const int64_t base = (int64_t)blockIdx.x * kTile;
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    const int64_t k = base + (int64_t)i * kThreads + threadIdx.x;
    if (k < n) atomicAdd(&h[(keys[k] >> shift) & (kDigits - 1)], 1u);
  }
  __syncthreads();
  hist[(int64_t)threadIdx.x * n_tiles + blockIdx.x] = (int32_t)h[threadIdx.x];
}

// vals_in == nullptr: the value of pair k is k itself (first pass of an argsort)
__global__ __launch_bounds__(kThreads) void radix_scatter(const uint32_t* __restrict__ keys_in,
                                                           const uint32_t* __restrict__ vals_in, int64_t n, int shift,
                                                           const int64_t* __restrict__ offs, int64_t n_tiles,
                                                           uint32_t* __restrict__ keys_out,
                                                           uint32_t* __restrict__ vals_out) {
  __shared__ uint32_t run[kWaves][kDigits];  // pairs with this digit in earlier wavefronts / earlier steps
  __shared__ int64_t first[kDigits];         // where the tile's first pair with this digit goes
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  first[threadIdx.x] = offs[(int64_t)threadIdx.x * n_tiles + blockIdx.x];
#pragma unroll
  for (int w = 0; w < kWaves; ++w) run[w][threadIdx.x] = 0u;
  __syncthreads();
  const int64_t wbase = (int64_t)blockIdx.x * kTile + (int64_t)wave * kWaveTile;
  uint32_t key[kWaveTile / 64];
#pragma unroll
  for (int c = 0; c < kWaveTile / 64; ++c) {
    const int64_t k = wbase + c * 64 + lane;
    key[c] = k < n ? keys_in[k] : 0u;
    if (k < n) atomicAdd(&run[wave][(key[c] >> shift) & (kDigits - 1)], 1u);
  }
  __syncthreads();
  {  // counts per wavefront -> counts in the wavefronts before it
    uint32_t before = 0u;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const uint32_t c = run[w][threadIdx.x];
      run[w][threadIdx.x] = before;
      before += c;
    }
  }
  __syncthreads();
  const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
  for (int c = 0; c < kWaveTile / 64; ++c) {
    const int64_t k = wbase + c * 64 + lane;
    const bool valid = k < n;
    const uint32_t d = (key[c] >> shift) & (kDigits - 1);
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const bool bit = (d >> b) & 1u;
      const uint64_t m = __ballot(valid && bit);
      peers &= bit ? m : ~m;
    }
    if (valid) {
      const uint32_t ahead = run[wave][d];  // read by every peer before the leader updates it below
      const int64_t dst = first[d] + ahead + (uint32_t)__popcll(peers & below);
      keys_out[dst] = key[c];
      vals_out[dst] = vals_in ? vals_in[k] : (uint32_t)k;
    }
    __builtin_amdgcn_wave_barrier();
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (valid && (peers & below) == 0ull) run[wave][d] += (uint32_t)__popcll(peers);  // one lane per digit value
    __builtin_amdgcn_wave_barrier();
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }
}

struct SortCarve {
  uint32_t *keys_alt, *vals_alt;
  int32_t* hist;
  int64_t* offs;
  int64_t* scan_tmp;
};

size_t carve_sort(int64_t n, void* tmp, SortCarve* out) {
  const int64_t n_tiles = std::max<int64_t>(ceil_div(n, kTile), 1);
  Carver c(tmp);
  SortCarve w;
  w.keys_alt = c.take<uint32_t>((size_t)std::max<int64_t>(n, 1));
  w.vals_alt = c.take<uint32_t>((size_t)std::max<int64_t>(n, 1));
  w.hist = c.take<int32_t>((size_t)(kDigits * n_tiles));
  w.offs = c.take<int64_t>((size_t)(kDigits * n_tiles) + 1);
  w.scan_tmp = c.take<int64_t>(scan_tmp_ints(kDigits * n_tiles));
  if (out) *out = w;
  return c.off;
}

}  // namespace

size_t radix_sort_tmp_bytes(int64_t n) { return carve_sort(std::max<int64_t>(n, 0), nullptr, nullptr); }

int radix_sort_pairs(const uint32_t* keys_in, const uint32_t* vals_in, uint32_t* keys_out, uint32_t* vals_out,
                     int64_t n, int key_bits, void* tmp, hipStream_t s) {
  if (n <= 0) return MGGCN_OK;
  MGGCN_REQUIRE(n < ((int64_t)1 << 32), MGGCN_E_OVERFLOW, "%lld pairs: positions are held in 32 unsigned bits", (long long)n);
  SortCarve w;
  carve_sort(n, tmp, &w);
  const int passes = std::max(1, (std::min(std::max(key_bits, 1), 32) + 7) / 8);
  const int64_t n_tiles = ceil_div(n, kTile);
  MGGCN_REQUIRE(n_tiles < ((int64_t)1 << 31), MGGCN_E_OVERFLOW, "sort grid too large");
  const uint32_t* kin = keys_in;
  const uint32_t* vin = vals_in;
  for (int p = 0; p < passes; ++p) {
    // the last pass writes the caller's arrays; the passes before it alternate between the two pairs of arrays
    const bool to_out = (passes - 1 - p) % 2 == 0;
    uint32_t* kout = to_out ? keys_out : w.keys_alt;
    uint32_t* vout = to_out ? vals_out : w.vals_alt;
    radix_hist<<<(unsigned)n_tiles, kThreads, 0, s>>>(kin, n, 8 * p, w.hist, n_tiles);
    MGGCN_LAUNCH_CHECK();
    const int rc = exclusive_scan_i64(w.hist, kDigits * n_tiles, w.offs, w.scan_tmp, s);
    if (rc) return rc;
    radix_scatter<<<(unsigned)n_tiles, kThreads, 0, s>>>(kin, vin, n, 8 * p, w.offs, n_tiles, kout, vout);
    MGGCN_LAUNCH_CHECK();
    kin = kout;
    vin = vout;
  }
  return MGGCN_OK;
}

}  // namespace mggcn
