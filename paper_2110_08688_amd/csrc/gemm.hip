// Dense fp32 GeMM on the CDNA matrix cores for the three products of a GCN layer
// (Eq. 5: H W, Eq. 10: H^T HW_G, Eq. 11: HW_G W^T of the paper).
//
//   C = epilogue( op(A) op(B) + beta C )
//
// Workgroups of 4 wavefronts own tiles of C and walk K in steps of 32 (16 for a short inner
// dimension); operand tiles are staged through LDS.  v_mfma_f32_32x32x2_f32 wants lane l to feed
// A[m = l%32][k = l/32] and B[k = l/32][n = l%32].
//   gemm_stream  operands whose rows start on 16-byte boundaries (every large product of a GCN
//                layer): buffer-addressed loads, two LDS stages, 128 x 128 tiles, several tiles
//                per workgroup;
//   gemm_mfma    everything else: 128 x 64 tiles, one LDS stage, checked loaders;
//   gemm_pieces  the same product out of bfloat16 matrix instructions (an extension).
// All three write C through the same epilogue (ReLU, ReLU' mask, beta = 1 fused).
//
// The shapes here are tall and skinny (M = vertex count, N and K a few hundred at most) except
// for the weight gradient, whose inner dimension is the vertex count: that one is split along
// K into partial products that a second kernel adds in split order (no
// floating-point atomics, so results are reproducible).
#include "common.h"

#include <algorithm>

namespace mggcn {
namespace {

constexpr int kThreads = 256;
constexpr int kXcds = 8;  // accelerator dies of an MI355X, each with its own L2

typedef float float16v __attribute__((ext_vector_type(16)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

// Buffer descriptor over `bytes` bytes at `base` (a value every lane agrees on): untyped 32-bit
// data, no stride.  A load through it takes its base from scalar registers and a 32-bit offset per
// lane, and returns 0 instead of touching memory at offsets of `bytes` or more; the range field
// has 32 bits, so longer ranges are cut to 4 GiB - 1 (a tile's own offsets stay far below that).
__device__ inline __amdgpu_buffer_rsrc_t buffer_over(const float* base, int64_t bytes) {
  const int64_t n = bytes < 0 ? 0 : (bytes > 0xffffffffll ? 0xffffffffll : bytes);
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(base), 0, (int)(uint32_t)n, 0x00020000);
}

// Tile of an operand whose memory rows run along K (A not transposed, or B transposed):
// R rows x BK, staged as 4 consecutive k per thread.
template <int R, int BK>
struct KContig {
  static constexpr int kThreadsPerRow = BK / 4;
  static constexpr int kRowsPerPass = kThreads / kThreadsPerRow;
  static constexpr int kPasses = R / kRowsPerPass;
  static constexpr int kRegs = kPasses * 4;
  static_assert(kPasses >= 1 && R % kRowsPerPass == 0, "tile does not divide over the workgroup");
  template <bool kFast>
  __device__ static inline void load(const float* __restrict__ src, int64_t ld, int64_t row0,
                                     int64_t row_end, int64_t k0, int64_t k_end, int vec,
                                     float (&reg)[kRegs]) {
    if (kFast || (row0 + R <= row_end && k0 + BK <= k_end)) {
      const int r = threadIdx.x / kThreadsPerRow, kq = threadIdx.x % kThreadsPerRow;
#pragma unroll
      for (int p = 0; p < kPasses; ++p) {  // interior tile: nothing to predicate
        const float* ptr = src + (row0 + p * kRowsPerPass + r) * ld + k0 + 4 * kq;
        if (vec == 4) {
          const float4 t = *reinterpret_cast<const float4*>(ptr);
          reg[p * 4 + 0] = t.x; reg[p * 4 + 1] = t.y; reg[p * 4 + 2] = t.z; reg[p * 4 + 3] = t.w;
        } else if (vec == 2) {  // rows aligned to 8 bytes only (odd multiples of two floats)
          const float2 t = *reinterpret_cast<const float2*>(ptr);
          const float2 u = *reinterpret_cast<const float2*>(ptr + 2);
          reg[p * 4 + 0] = t.x; reg[p * 4 + 1] = t.y; reg[p * 4 + 2] = u.x; reg[p * 4 + 3] = u.y;
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i) reg[p * 4 + i] = ptr[i];
        }
      }
      return;
    }
    const int r = threadIdx.x / kThreadsPerRow, kq = threadIdx.x % kThreadsPerRow;
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
      const int64_t row = row0 + p * kRowsPerPass + r;
      const int64_t k = k0 + 4 * kq;
      const float* ptr = src + row * ld + k;
      if (vec == 4 && row < row_end && k + 3 < k_end) {
        const float4 t = *reinterpret_cast<const float4*>(ptr);
        reg[p * 4 + 0] = t.x; reg[p * 4 + 1] = t.y; reg[p * 4 + 2] = t.z; reg[p * 4 + 3] = t.w;
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) reg[p * 4 + i] = (row < row_end && k + i < k_end) ? ptr[i] : 0.f;
      }
    }
  }
  template <int LD>
  __device__ static inline void store(float (*S)[LD], const float (&reg)[kRegs]) {
    const int r = threadIdx.x / kThreadsPerRow, kq = threadIdx.x % kThreadsPerRow;
#pragma unroll
    for (int p = 0; p < kPasses; ++p)
#pragma unroll
      for (int i = 0; i < 4; ++i) S[4 * kq + i][p * kRowsPerPass + r] = reg[p * 4 + i];
  }
  // The tile as it lies in memory, S[row][k]: one 16-byte store per piece.
  template <int LD>
  __device__ static inline void store_rows(float (*S)[LD], const float (&reg)[kRegs]) {
    static_assert(LD % 4 == 0, "row stride must keep 16-byte alignment");
    const int r = threadIdx.x / kThreadsPerRow, kq = threadIdx.x % kThreadsPerRow;
#pragma unroll
    for (int p = 0; p < kPasses; ++p)
      *reinterpret_cast<float4*>(&S[p * kRowsPerPass + r][4 * kq]) =
          make_float4(reg[p * 4 + 0], reg[p * 4 + 1], reg[p * 4 + 2], reg[p * 4 + 3]);
  }
  // Byte offsets of this thread's 16-byte pieces from the tile's corner; they do not change along K.
  __device__ static inline void offsets(int64_t ld, uint32_t (&off)[kPasses]) {
    const int r = threadIdx.x / kThreadsPerRow, kq = threadIdx.x % kThreadsPerRow;
#pragma unroll
    for (int p = 0; p < kPasses; ++p) off[p] = (uint32_t)(((int64_t)(p * kRowsPerPass + r) * ld + 4 * kq) * 4);
  }
  // A whole k-step through the buffer path: the base is the tile's corner at column k0 (scalar
  // registers), the hardware returns 0 for anything past the last valid byte of the matrix, so the
  // rows of a ragged last tile need no test.  k0 + BK <= n_k.
  __device__ static inline void load_buffer(const float* __restrict__ src, int64_t ld, int64_t row0, int64_t row_end,
                                            int64_t k0, int64_t n_k, const uint32_t (&off)[kPasses],
                                            float (&reg)[kRegs]) {
    const __amdgpu_buffer_rsrc_t rs =
        buffer_over(src + row0 * ld + k0, ((row_end - row0 - 1) * ld + (n_k - k0)) * (int64_t)sizeof(float));
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
      const uint4v t = __builtin_amdgcn_raw_buffer_load_b128(rs, off[p], 0, 0);
      reg[p * 4 + 0] = __uint_as_float(t.x); reg[p * 4 + 1] = __uint_as_float(t.y);
      reg[p * 4 + 2] = __uint_as_float(t.z); reg[p * 4 + 3] = __uint_as_float(t.w);
    }
  }
};

// Tile of an operand whose memory rows run along the tile's M/N side (A transposed, or B not
// transposed): BK x R, 4 consecutive m (or n) per thread.
template <int R, int BK>
struct MContig {
  static constexpr int kThreadsPerRow = R / 4;
  static constexpr int kRowsPerPass = kThreads / kThreadsPerRow;
  static constexpr int kPasses = BK / kRowsPerPass;
  static constexpr int kRegs = kPasses * 4;
  static_assert(kPasses >= 1 && BK % kRowsPerPass == 0, "tile does not divide over the workgroup");
  template <bool kFast>
  __device__ static inline void load(const float* __restrict__ src, int64_t ld, int64_t col0,
                                     int64_t col_end, int64_t k0, int64_t k_end, int vec,
                                     float (&reg)[kRegs]) {
    if (kFast || (col0 + R <= col_end && k0 + BK <= k_end)) {
      const int cq = threadIdx.x % kThreadsPerRow, kr = threadIdx.x / kThreadsPerRow;
#pragma unroll
      for (int p = 0; p < kPasses; ++p) {  // interior tile: nothing to predicate
        const float* ptr = src + (k0 + p * kRowsPerPass + kr) * ld + col0 + 4 * cq;
        if (vec == 4) {
          const float4 t = *reinterpret_cast<const float4*>(ptr);
          reg[p * 4 + 0] = t.x; reg[p * 4 + 1] = t.y; reg[p * 4 + 2] = t.z; reg[p * 4 + 3] = t.w;
        } else if (vec == 2) {  // rows aligned to 8 bytes only (odd multiples of two floats)
          const float2 t = *reinterpret_cast<const float2*>(ptr);
          const float2 u = *reinterpret_cast<const float2*>(ptr + 2);
          reg[p * 4 + 0] = t.x; reg[p * 4 + 1] = t.y; reg[p * 4 + 2] = u.x; reg[p * 4 + 3] = u.y;
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i) reg[p * 4 + i] = ptr[i];
        }
      }
      return;
    }
    const int cq = threadIdx.x % kThreadsPerRow, kr = threadIdx.x / kThreadsPerRow;
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
      const int64_t k = k0 + p * kRowsPerPass + kr;
      const int64_t col = col0 + 4 * cq;
      const float* ptr = src + k * ld + col;
      if (vec == 4 && k < k_end && col + 3 < col_end) {
        const float4 t = *reinterpret_cast<const float4*>(ptr);
        reg[p * 4 + 0] = t.x; reg[p * 4 + 1] = t.y; reg[p * 4 + 2] = t.z; reg[p * 4 + 3] = t.w;
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) reg[p * 4 + i] = (k < k_end && col + i < col_end) ? ptr[i] : 0.f;
      }
    }
  }
  template <int LD>
  __device__ static inline void store(float (*S)[LD], const float (&reg)[kRegs]) {
    static_assert(LD % 4 == 0, "row stride must keep 16-byte alignment");
    const int cq = threadIdx.x % kThreadsPerRow, kr = threadIdx.x / kThreadsPerRow;
#pragma unroll
    for (int p = 0; p < kPasses; ++p)
      *reinterpret_cast<float4*>(&S[p * kRowsPerPass + kr][4 * cq]) =
          make_float4(reg[p * 4 + 0], reg[p * 4 + 1], reg[p * 4 + 2], reg[p * 4 + 3]);
  }
  __device__ static inline void offsets(int64_t ld, uint32_t (&off)[kPasses]) {
    const int cq = threadIdx.x % kThreadsPerRow, kr = threadIdx.x / kThreadsPerRow;
#pragma unroll
    for (int p = 0; p < kPasses; ++p) off[p] = (uint32_t)(((int64_t)(p * kRowsPerPass + kr) * ld + 4 * cq) * 4);
  }
  // As above; memory rows run along the tile's M/N side here, so the base moves down BK rows per
  // k-step.  Columns past col_end of a ragged tile read the neighbouring row (finite or not, they
  // only reach accumulators that are never stored) except in the matrix's last row, where the
  // range check returns 0.  k0 + BK <= n_k.
  __device__ static inline void load_buffer(const float* __restrict__ src, int64_t ld, int64_t col0, int64_t col_end,
                                            int64_t k0, int64_t n_k, const uint32_t (&off)[kPasses],
                                            float (&reg)[kRegs]) {
    const __amdgpu_buffer_rsrc_t rs =
        buffer_over(src + k0 * ld + col0, ((n_k - k0 - 1) * ld + (col_end - col0)) * (int64_t)sizeof(float));
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
      const uint4v t = __builtin_amdgcn_raw_buffer_load_b128(rs, off[p], 0, 0);
      reg[p * 4 + 0] = __uint_as_float(t.x); reg[p * 4 + 1] = __uint_as_float(t.y);
      reg[p * 4 + 2] = __uint_as_float(t.z); reg[p * 4 + 3] = __uint_as_float(t.w);
    }
  }
};

__device__ inline float gemm_epilogue(float acc, float old, float beta, int epi) {
  if (beta != 0.f) acc += old;
  if (epi == MGGCN_EPI_RELU) acc = acc > 0.f ? acc : 0.f;
  if (epi == MGGCN_EPI_RELU_MASK) acc = old > 0.f ? acc : 0.f;
  return acc;
}

// Workgroups are dealt to the 8 XCDs round-robin by index, and each XCD has its own L2.  The
// 1-D grid is therefore decoded so that the N tiles of one M tile -- they re-read the same rows
// of A -- sit on one XCD next to each other in time.  Measured on 2.45M x 256 x 256: 3.33 ->
// 2.91 ms, A being fetched from HBM once instead of four times.  With a split inner dimension
// the tiles of a split read disjoint columns of A, and the plain order (M tiles fastest, spread
// over the XCDs) measured faster than grouping a split on one XCD.
// Returns false for a workgroup that only pads the grid to whole groups of 8.
__device__ inline bool decode_tile(int64_t m_rows, int64_t N, int64_t K, int bm, int bn, int64_t k_per_split,
                                   int64_t* tile_m, int64_t* tile_n, int64_t* split) {
  const int64_t tiles_m = (m_rows + bm - 1) / bm, tiles_n = (N + bn - 1) / bn;
  const int64_t splits = (K + k_per_split - 1) / k_per_split;
  if (splits == 1) {
    const int64_t xcd = blockIdx.x % kXcds, local = blockIdx.x / kXcds;
    *tile_n = local % tiles_n;
    *tile_m = (local / tiles_n) * kXcds + xcd;
    *split = 0;
    return *tile_m < tiles_m;
  }
  const int64_t per = tiles_m * tiles_n, t = blockIdx.x % per;
  *split = blockIdx.x / per;
  *tile_m = t % tiles_m;
  *tile_n = t / tiles_m;
  return true;
}

// The TM x TN accumulator tiles of one wavefront, whose corner is (row0, col0), go to C (with the
// epilogue) or to this split's partial product.  Accumulator register r of lane l is
// C[8*(r/4) + 4*(l/32) + r%4][l%32] of its 32x32 tile.
template <int TM, int TN>
__device__ inline void store_tiles(const float16v (&acc)[TM][TN], int64_t row0, int64_t col0, bool whole, int64_t M,
                                   int64_t N, int64_t split, float* __restrict__ C, int64_t ldc, float beta,
                                   int epi, float* __restrict__ partial) {
  const int lane = threadIdx.x & 63;
  const int frow = lane >> 5, fcol = lane & 31;
  const bool to_partial = partial != nullptr;
  float* out = to_partial ? partial + split * M * N : C;
  const int64_t ldo = to_partial ? N : ldc;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int64_t col = col0 + j * 32 + fcol;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t row = row0 + i * 32 + 8 * (r / 4) + 4 * frow + (r % 4);
        if (whole || (row < M && col < N)) {
          float* dst = out + row * ldo + col;
          if (to_partial) {
            *dst = acc[i][j][r];
          } else {
            const float old = (beta != 0.f || epi == MGGCN_EPI_RELU_MASK) ? *dst : 0.f;
            *dst = gemm_epilogue(acc[i][j][r], old, beta, epi);
          }
        }
      }
    }
}

// The same for a wavefront whose TM x TN tiles lie wholly inside C: no test per element, and no
// vector arithmetic for addresses -- one buffer descriptor over the wavefront's block, one offset
// per lane, and the offset of each accumulator register's row in a scalar register.
template <int TM, int TN>
__device__ inline void store_whole_tiles(const float16v (&acc)[TM][TN], int64_t row0, int64_t col0, int64_t M,
                                         int64_t N, int64_t split, float* __restrict__ C, int64_t ldc, float beta,
                                         int epi, float* __restrict__ partial) {
  const int lane = threadIdx.x & 63;
  const int frow = lane >> 5, fcol = lane & 31;
  const bool to_partial = partial != nullptr;
  float* out = to_partial ? partial + split * M * N : C;
  const int64_t ldo = to_partial ? N : ldc;
  const __amdgpu_buffer_rsrc_t rs =
      buffer_over(out + row0 * ldo + col0, ((TM * 32 - 1) * ldo + TN * 32) * (int64_t)sizeof(float));
  const uint32_t lane_off = (uint32_t)((4 * frow * ldo + fcol) * 4);
  // the choice is the same for every element: made once, outside the unrolled stores
  auto sweep = [&](auto mode) {
    constexpr int kMode = decltype(mode)::value;  // 0: as it is, 1: ReLU, 2: needs the old value of C
    // the old values of one 32 x 32 tile are all requested before the first of them is used: one
    // memory latency per tile instead of one per element (loads and stores through one descriptor
    // are not reordered by the compiler)
    float old[kMode == 2 ? 16 : 1];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        if constexpr (kMode == 2) {
#pragma unroll
          for (int r = 0; r < 16; ++r)
            old[r] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(
                rs, lane_off, (uint32_t)(((i * 32 + 8 * (r / 4) + (r % 4)) * ldo + j * 32) * 4), 0));
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const uint32_t reg_off = (uint32_t)(((i * 32 + 8 * (r / 4) + (r % 4)) * ldo + j * 32) * 4);
          float v = acc[i][j][r];
          if constexpr (kMode == 1) v = v > 0.f ? v : 0.f;
          if constexpr (kMode == 2) v = gemm_epilogue(v, old[r], beta, epi);
          __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), rs, lane_off, reg_off, 0);
        }
      }
  };
  if (to_partial || (beta == 0.f && epi == MGGCN_EPI_NONE)) sweep(std::integral_constant<int, 0>{});
  else if (beta == 0.f && epi == MGGCN_EPI_RELU) sweep(std::integral_constant<int, 1>{});
  else sweep(std::integral_constant<int, 2>{});
}

// And for a wavefront at the edge of C: columns past N are masked once per 32-column tile, rows
// past M fall outside the buffer descriptor (which ends with the last valid element) and are
// dropped by its range check; the row part of the offset is then per lane (one addition per store).
template <int TM, int TN>
__device__ inline void store_edge_tiles(const float16v (&acc)[TM][TN], int64_t row0, int64_t col0, int64_t M,
                                        int64_t N, int64_t split, float* __restrict__ C, int64_t ldc, float beta,
                                        int epi, float* __restrict__ partial) {
  if (row0 >= M || col0 >= N) return;
  const int lane = threadIdx.x & 63;
  const int frow = lane >> 5, fcol = lane & 31;
  const bool to_partial = partial != nullptr;
  float* out = to_partial ? partial + split * M * N : C;
  const int64_t ldo = to_partial ? N : ldc;
  const __amdgpu_buffer_rsrc_t rs =
      buffer_over(out + row0 * ldo + col0, ((M - row0 - 1) * ldo + (N - col0)) * (int64_t)sizeof(float));
  const uint32_t lane_off = (uint32_t)((4 * frow * ldo + fcol) * 4);
  auto sweep = [&](auto mode) {
    constexpr int kMode = decltype(mode)::value;
    float old[kMode == 2 ? 16 : 1];  // requested together, as above
#pragma unroll
    for (int j = 0; j < TN; ++j)
      if (col0 + j * 32 + fcol < N) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          if constexpr (kMode == 2) {
#pragma unroll
            for (int r = 0; r < 16; ++r)
              old[r] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(
                  rs, lane_off + (uint32_t)(((i * 32 + 8 * (r / 4) + (r % 4)) * ldo + j * 32) * 4), 0, 0));
          }
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const uint32_t off = lane_off + (uint32_t)(((i * 32 + 8 * (r / 4) + (r % 4)) * ldo + j * 32) * 4);
            float v = acc[i][j][r];
            if constexpr (kMode == 1) v = v > 0.f ? v : 0.f;
            if constexpr (kMode == 2) v = gemm_epilogue(v, old[r], beta, epi);
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), rs, off, 0, 0);
          }
        }
      }
  };
  if (to_partial || (beta == 0.f && epi == MGGCN_EPI_NONE)) sweep(std::integral_constant<int, 0>{});
  else if (beta == 0.f && epi == MGGCN_EPI_RELU) sweep(std::integral_constant<int, 1>{});
  else sweep(std::integral_constant<int, 2>{});
}

// per-lane byte offsets inside a wavefront's block of C stay below 2^31 for rows shorter than this
constexpr int64_t kBufferMaxLd = (int64_t)1 << 21;

// row0, col0 and everything else but the accumulators must be the same in all lanes.
template <int TM, int TN>
__device__ inline void write_tiles(const float16v (&acc)[TM][TN], int64_t row0, int64_t col0, int64_t M, int64_t N,
                                   int64_t split, float* __restrict__ C, int64_t ldc, float beta, int epi,
                                   float* __restrict__ partial) {
  const int64_t ldo = partial ? N : ldc;
  if (ldo >= kBufferMaxLd) store_tiles<TM, TN>(acc, row0, col0, false, M, N, split, C, ldc, beta, epi, partial);
  else if (row0 + TM * 32 <= M && col0 + TN * 32 <= N)
    store_whole_tiles<TM, TN>(acc, row0, col0, M, N, split, C, ldc, beta, epi, partial);
  else store_edge_tiles<TM, TN>(acc, row0, col0, M, N, split, C, ldc, beta, epi, partial);
}

// WM x WN wavefronts tile the BM x BN block; each wavefront holds TM x TN accumulators of 32x32.
// kFast: the host guarantees 16-byte aligned operands and whole tiles along N, so a block whose
// M tile is whole loads its full k-steps with no checks at all (measured +15 %); the ragged last
// row tile and a ragged last k-step go through the checked loader.
template <int BM, int BN, int BK, int WM, int WN, bool TA, bool TB, bool kFast>
__global__ __launch_bounds__(kThreads) void gemm_mfma(int64_t m_base, int64_t M, int64_t N, int64_t K,
                                                       const float* __restrict__ A, int64_t lda,
                                                       const float* __restrict__ B, int64_t ldb,
                                                       float* __restrict__ C, int64_t ldc, float beta,
                                                       int epi, int64_t k_per_split,
                                                       float* __restrict__ partial, int vecA,
                                                       int vecB) {
  static_assert(WM * WN == kThreads / 64, "four wavefronts");
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  static_assert(TM >= 1 && TN >= 1, "wave tile must hold at least one 32x32 MFMA tile");
  // row padding: 16-byte aligned rows for the vector stores of an m-contiguous operand; for the
  // transposing scalar stores of a k-contiguous one, the stride that spreads the BK/4 k-quads of a
  // half-wavefront over distinct banks
  constexpr int LDA = BM + (TA ? 4 : 32 / BK);
  constexpr int LDB = BN + (TB ? 32 / BK : 4);
  using LoadA = typename std::conditional<TA, MContig<BM, BK>, KContig<BM, BK>>::type;
  using LoadB = typename std::conditional<TB, KContig<BN, BK>, MContig<BN, BK>>::type;

  __shared__ __attribute__((aligned(16))) float As[BK][LDA];
  __shared__ __attribute__((aligned(16))) float Bs[BK][LDB];

  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // a scalar
  const int wm = wave / WN, wn = wave % WN;
  int64_t tile_m, tile_n, split;
  if (!decode_tile(M - m_base, N, K, BM, BN, k_per_split, &tile_m, &tile_n, &split)) return;
  const int64_t m0 = m_base + tile_m * BM;
  const int64_t n0 = tile_n * BN;
  const int64_t kb = split * k_per_split;
  const int64_t ke = min(K, kb + k_per_split);

  float16v acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  float ra[LoadA::kRegs], rb[LoadB::kRegs];
  const bool whole = kFast && m0 + BM <= M;  // uniform over the block
  auto load_step = [&](int64_t k) {
    if (whole && k + BK <= ke) {
      LoadA::template load<true>(A, lda, m0, M, k, ke, 4, ra);
      LoadB::template load<true>(B, ldb, n0, N, k, ke, 4, rb);
    } else {
      LoadA::template load<false>(A, lda, m0, M, k, ke, vecA, ra);
      LoadB::template load<false>(B, ldb, n0, N, k, ke, vecB, rb);
    }
  };
  load_step(kb);

  const int frow = lane >> 5, fcol = lane & 31;
  for (int64_t k0 = kb; k0 < ke; k0 += BK) {
    LoadA::template store<LDA>(As, ra);
    LoadB::template store<LDB>(Bs, rb);
    __syncthreads();
    if (k0 + BK < ke) load_step(k0 + BK);  // in flight during the MFMA loop below
    // all fragments of the step are read from LDS first, then the MFMAs run back to back
    float a[BK / 2][TM], b[BK / 2][TN];
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
#pragma unroll
      for (int i = 0; i < TM; ++i) a[kk / 2][i] = As[kk + frow][(wm * TM + i) * 32 + fcol];
#pragma unroll
      for (int j = 0; j < TN; ++j) b[kk / 2][j] = Bs[kk + frow][(wn * TN + j) * 32 + fcol];
    }
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[kk / 2][i], b[kk / 2][j], acc[i][j], 0, 0, 0);
    // ask the scheduler for LDS reads that run a few k-pairs ahead of the MFMAs consuming them
    __builtin_amdgcn_sched_group_barrier(0x100, 4 * 2, 0);
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
      __builtin_amdgcn_sched_group_barrier(0x008, TM * TN, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    }
    __syncthreads();
  }

  write_tiles<TM, TN>(acc, m0 + wm * TM * 32, n0 + wn * TN * 32, M, N, split, C, ldc, beta, epi, partial);
}


// The same product for the shapes that carry the time: 16-byte aligned rows and whole tiles
// along N (the host checks both).  What differs from gemm_mfma:
//   * operands travel global -> registers through buffer loads whose base lives in scalar
//     registers and whose per-lane offsets are fixed for the whole tile, so that a k-step issues
//     no vector arithmetic for addresses (vector instructions take issue slots from the matrix
//     pipe of the same SIMD), and a ragged last row tile is handled by the range check of the
//     descriptor instead of predicates;
//   * two LDS stages and one barrier per k-step: the loads of step s+1 are issued before the
//     matrix instructions of step s and written to the other stage after them;
//   * for N a multiple of 128 the tile is 128 x 128 with 64 x 64 per wavefront: one LDS read per
//     matrix instruction instead of 1.5 and two thirds of the global bytes per flop.  On this
//     chip that is what decides the speed on real data: the same instruction stream runs
//     ~20 % slower on random operands than on constant ones with 32 x 64 per wavefront (the
//     clock is lowered under the switching activity of LDS, load path and matrix pipes
//     together) and ~5 % slower with 64 x 64.
// A ragged last k-step goes through the checked loaders of gemm_mfma.
// Where a workgroup's next tile is.  Virtual workgroup ids follow decode_tile's order (unsplit: the N
// tiles of an M tile next to each other on one XCD; ids that only pad the grid to whole groups of
// 8 M tiles are skipped), and a workgroup takes the ids blockIdx.x, blockIdx.x + gridDim.x, ...:
// with a grid that is a multiple of 8 it stays on its XCD's share of the tiles.
struct TilePos {
  uint32_t id;
  int64_t m0, n0, kb, ke;
  int64_t split, steps, whole_steps;
};

__device__ inline bool locate_tile(uint32_t id, uint32_t n_ids, uint32_t stride, uint32_t tiles_m, uint32_t tiles_n,
                                   uint32_t splits, int64_t K, int64_t k_per_split, int bm, int bn, int bk,
                                   TilePos* pos) {
  for (; id < n_ids; id += stride) {
    uint32_t tm, tn, split;
    if (splits == 1) {
      const uint32_t xcd = id % kXcds, local = id / kXcds;
      tn = local % tiles_n;
      tm = (local / tiles_n) * kXcds + xcd;
      split = 0;
      if (tm >= tiles_m) continue;
    } else {
      const uint32_t per = tiles_m * tiles_n, t = id % per;
      split = id / per;
      tm = t % tiles_m;
      tn = t / tiles_m;
    }
    pos->id = id;
    pos->m0 = (int64_t)tm * bm;
    pos->n0 = (int64_t)tn * bn;
    pos->split = split;
    pos->kb = (int64_t)split * k_per_split;
    pos->ke = min(K, pos->kb + k_per_split);
    pos->steps = (pos->ke - pos->kb + bk - 1) / bk;
    pos->whole_steps = (pos->ke - pos->kb) / bk;
    return true;
  }
  return false;
}

template <int BN, int WM, int WN, bool TA, bool TB>
__global__ __launch_bounds__(kThreads, 2) void gemm_stream(int64_t M, int64_t N, int64_t K,
                                                         const float* __restrict__ A, int64_t lda,
                                                         const float* __restrict__ B, int64_t ldb,
                                                         float* __restrict__ C, int64_t ldc, float beta, int epi,
                                                         int64_t k_per_split, float* __restrict__ partial,
                                                         uint32_t n_ids, uint32_t tiles_m, uint32_t tiles_n,
                                                         uint32_t splits) {
  static_assert(WM * WN == kThreads / 64, "four wavefronts");
  constexpr int BM = 128, BK = 32, TM = BM / WM / 32, TN = BN / WN / 32;
  // An operand whose memory rows run along K keeps that order in LDS, S[m][k] with rows of 36
  // floats: 16-byte stores, and a fragment is one 16-byte read per four matrix instructions (16
  // neighbouring lanes fall on 64 distinct banks).  The other kind is staged k-major, S[k][m], and
  // read 4 bytes at a time.  Lane l of matrix instruction t of the q-th group of eight k feeds
  // k = 8q + 4(l/32) + t for both operands, which is the order the 16-byte reads deliver.
  constexpr bool kRowsA = !TA, kRowsB = TB;
  constexpr int LDA = kRowsA ? BK + 4 : BM + 4;
  constexpr int LDB = kRowsB ? BK + 4 : BN + 4;
  using LoadA = typename std::conditional<TA, MContig<BM, BK>, KContig<BM, BK>>::type;
  using LoadB = typename std::conditional<TB, KContig<BN, BK>, MContig<BN, BK>>::type;

  __shared__ __attribute__((aligned(16))) float As[2][kRowsA ? BM : BK][LDA];
  __shared__ __attribute__((aligned(16))) float Bs[2][kRowsB ? BN : BK][LDB];

  // the wavefront's number as a scalar: what depends on it (its corner of the tile, the buffer
  // descriptor of its part of C) then lives in scalar registers
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / WN, wn = wave % WN;
  TilePos cur;
  if (!locate_tile(blockIdx.x, n_ids, gridDim.x, tiles_m, tiles_n, splits, K, k_per_split, BM, BN, BK, &cur)) return;

  float16v acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  uint32_t offA[LoadA::kPasses], offB[LoadB::kPasses];
  LoadA::offsets(lda, offA);
  LoadB::offsets(ldb, offB);
  float ra[LoadA::kRegs], rb[LoadB::kRegs];
  auto load_step = [&](const TilePos& t, int64_t s) {
    const int64_t k = t.kb + s * BK;
    if (s < t.whole_steps) {
      LoadA::load_buffer(A, lda, t.m0, M, k, K, offA, ra);
      LoadB::load_buffer(B, ldb, t.n0, N, k, K, offB, rb);
    } else {
      LoadA::template load<false>(A, lda, t.m0, M, k, t.ke, 4, ra);
      LoadB::template load<false>(B, ldb, t.n0, N, k, t.ke, 4, rb);
    }
  };
  const int frow = lane >> 5, fcol = lane & 31;
  auto stage_tiles = [&](int stage) {
    if constexpr (kRowsA) LoadA::template store_rows<LDA>(As[stage], ra);
    else LoadA::template store<LDA>(As[stage], ra);
    if constexpr (kRowsB) LoadB::template store_rows<LDB>(Bs[stage], rb);
    else LoadB::template store<LDB>(Bs[stage], rb);
  };
  auto multiply = [&](int stage) {
    float a[BK / 2][TM], b[BK / 2][TN];
#pragma unroll
    for (int q = 0; q < BK / 8; ++q) {
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        if constexpr (kRowsA) {
          const float4 v = *reinterpret_cast<const float4*>(&As[stage][(wm * TM + i) * 32 + fcol][8 * q + 4 * frow]);
          a[4 * q + 0][i] = v.x; a[4 * q + 1][i] = v.y; a[4 * q + 2][i] = v.z; a[4 * q + 3][i] = v.w;
        } else {
#pragma unroll
          for (int t = 0; t < 4; ++t) a[4 * q + t][i] = As[stage][8 * q + 4 * frow + t][(wm * TM + i) * 32 + fcol];
        }
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        if constexpr (kRowsB) {
          const float4 v = *reinterpret_cast<const float4*>(&Bs[stage][(wn * TN + j) * 32 + fcol][8 * q + 4 * frow]);
          b[4 * q + 0][j] = v.x; b[4 * q + 1][j] = v.y; b[4 * q + 2][j] = v.z; b[4 * q + 3][j] = v.w;
        } else {
#pragma unroll
          for (int t = 0; t < 4; ++t) b[4 * q + t][j] = Bs[stage][8 * q + 4 * frow + t][(wn * TN + j) * 32 + fcol];
        }
      }
    }
#pragma unroll
    for (int kk = 0; kk < BK / 2; ++kk)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[kk][i], b[kk][j], acc[i][j], 0, 0, 0);
    // LDS reads one group of eight k ahead of the matrix instructions that consume them
    constexpr int kReads = (kRowsA ? TM : 4 * TM) + (kRowsB ? TN : 4 * TN);  // per group of eight k
    __builtin_amdgcn_sched_group_barrier(0x100, kReads, 0);
#pragma unroll
    for (int q = 0; q < BK / 8; ++q)
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        __builtin_amdgcn_sched_group_barrier(0x008, TM * TN, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, (kReads + 3) / 4, 0);
      }
  };

  load_step(cur, 0);
  stage_tiles(0);
  __syncthreads();
  int stage = 0;
  for (;;) {
    // all k-steps of the tile but the last: the accumulators see nothing but matrix instructions
    for (int64_t s = 0; s + 1 < cur.steps; ++s) {
      load_step(cur, s + 1);  // in flight during the matrix instructions below
      multiply(stage);
      stage_tiles(stage ^ 1);
      __syncthreads();  // the other stage is complete, and everyone is done reading this one
      stage ^= 1;
    }
    // the last one: the first operands of the workgroup's next tile are on their way while this
    // tile's result is written
    TilePos nxt;
    const bool more =
        locate_tile(cur.id + gridDim.x, n_ids, gridDim.x, tiles_m, tiles_n, splits, K, k_per_split, BM, BN, BK, &nxt);
    if (more) load_step(nxt, 0);
    multiply(stage);
    write_tiles<TM, TN>(acc, cur.m0 + wm * TM * 32, cur.n0 + wn * TN * 32, M, N, cur.split, C, ldc, beta, epi, partial);
    if (!more) break;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    stage_tiles(stage ^ 1);
    __syncthreads();
    stage ^= 1;
    cur = nxt;
  }
}


// ---------------------------------------------------------------------------------------
// fp32 products out of bfloat16 matrix instructions
// ---------------------------------------------------------------------------------------
// An fp32 number is the exact sum of three bfloat16 numbers: its upper 16 bits, the upper 16 bits
// of what that leaves, and the rest (24 significand bits = 3 x 8, every difference exact).  With
// a = a0 + a1 + a2 and b = b0 + b1 + b2 the product a b is the sum of nine piece products, each of
// which the bf16 matrix instruction forms exactly and adds in fp32.  With |a1| < 2^-7 |a| and
// |a2| < 2^-15 |a| (2^-8 and 2^-16 on average) the three smallest, a1 b2 + a2 b1 + a2 b2, stay
// below 2^-21 |a b| (about 2^-24 |a b| on average: one fp32 rounding of the product) and are
// dropped; unlike the rounding of the running sum, which fp32 arithmetic of any kind pays at
// every one of the K additions, this error does not grow with K.  The other six are added
// smallest first.  Six v_mfma_f32_32x32x16_bf16 do the
// work of eight v_mfma_f32_32x32x2_f32 in a quarter of their time, so the product runs at up to
// 2.6x the fp32 matrix rate; the price is the split itself (5.5 vector operations per element
// staged, done once per tile) and 1.5x the LDS traffic.
// Non-finite inputs: a piece of Inf is Inf and leaves Inf - Inf, so an Inf operand yields NaN where
// fp32 arithmetic yields Inf; NaN stays NaN.  Values below 2^-110 lose their lower pieces to the
// subnormal flush of the matrix unit (absolute error below 2^-126 per product).
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kPieceBK = 32;
// 80-byte rows: the 16-byte fragment reads of 32 consecutive rows fall on distinct banks, and so
// do the 8-byte stores of the loaders (two rows of 64 bytes per 32 lanes)
constexpr int kPieceLd = kPieceBK + 8;

// upper halves of two words: (lo >> 16) | (hi & 0xffff0000)
__device__ inline uint32_t upper_halves(uint32_t hi, uint32_t lo) { return __builtin_amdgcn_perm(hi, lo, 0x07060302u); }

// Four values that follow each other along k, cut into their three pieces and stored as four
// bfloat16 per piece plane at S[plane][row][k4 .. k4+3].
template <int R>
__device__ inline void store_pieces(uint16_t (*S)[R][kPieceLd], int row, int k4, float x0, float x1, float x2,
                                    float x3) {
  const float x[4] = {x0, x1, x2, x3};
  uint32_t top[4], mid[4], low[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    top[i] = __float_as_uint(x[i]);
    const float r1 = x[i] - __uint_as_float(top[i] & 0xffff0000u);  // exact: at most 16 significant bits left
    mid[i] = __float_as_uint(r1);
    const float r2 = r1 - __uint_as_float(mid[i] & 0xffff0000u);    // exact: at most 8 left, a bfloat16 as it is
    low[i] = __float_as_uint(r2);
  }
  *reinterpret_cast<uint2*>(&S[0][row][k4]) = make_uint2(upper_halves(top[1], top[0]), upper_halves(top[3], top[2]));
  *reinterpret_cast<uint2*>(&S[1][row][k4]) = make_uint2(upper_halves(mid[1], mid[0]), upper_halves(mid[3], mid[2]));
  *reinterpret_cast<uint2*>(&S[2][row][k4]) = make_uint2(upper_halves(low[1], low[0]), upper_halves(low[3], low[2]));
}

// Staging of a tile whose memory rows run along K (see KContig, whose loads are used): thread
// (row r, k-quad kq) of each pass holds four consecutive k of one row.
template <int R>
__device__ inline void store_pieces_kcontig(uint16_t (*S)[R][kPieceLd], const float (&reg)[KContig<R, kPieceBK>::kRegs]) {
  using L = KContig<R, kPieceBK>;
  const int r = threadIdx.x / L::kThreadsPerRow, kq = threadIdx.x % L::kThreadsPerRow;
#pragma unroll
  for (int p = 0; p < L::kPasses; ++p)
    store_pieces<R>(S, p * L::kRowsPerPass + r, 4 * kq, reg[p * 4 + 0], reg[p * 4 + 1], reg[p * 4 + 2], reg[p * 4 + 3]);
}

// Tile of an operand whose memory rows run along the tile's M/N side, 32 x R: a thread takes a
// 4 x 4 block -- four consecutive k (one load each) of four consecutive columns -- so that after
// the transposition in registers every column again has four consecutive k to store.  Lanes run
// along k first (8 groups of 4), then along the column quads: one load instruction reads eight
// whole 128-byte lines.  R / 4 * 8 threads take part.
template <int R>
struct MContigK4 {
  static constexpr int kUsed = R / 4 * 8;
  static constexpr int kRegs = 16;
  static_assert(kUsed <= kThreads, "tile wider than the workgroup can stage");
  template <bool kFast>
  __device__ static inline void load(const float* __restrict__ src, int64_t ld, int64_t col0, int64_t col_end,
                                     int64_t k0, int64_t k_end, int vec, float (&reg)[kRegs]) {
    const int kg = threadIdx.x % 8, cq = threadIdx.x / 8;
    if (kUsed < kThreads && threadIdx.x >= kUsed) return;
    const int64_t col = col0 + 4 * cq;
    const bool interior = kFast || (col0 + R <= col_end && k0 + kPieceBK <= k_end);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const int64_t k = k0 + 4 * kg + p;
      const float* ptr = src + k * ld + col;
      if (interior && vec == 4) {
        const float4 t = *reinterpret_cast<const float4*>(ptr);
        reg[p * 4 + 0] = t.x; reg[p * 4 + 1] = t.y; reg[p * 4 + 2] = t.z; reg[p * 4 + 3] = t.w;
      } else if (interior && vec == 2) {
        const float2 t = *reinterpret_cast<const float2*>(ptr);
        const float2 u = *reinterpret_cast<const float2*>(ptr + 2);
        reg[p * 4 + 0] = t.x; reg[p * 4 + 1] = t.y; reg[p * 4 + 2] = u.x; reg[p * 4 + 3] = u.y;
      } else if (interior) {
#pragma unroll
        for (int i = 0; i < 4; ++i) reg[p * 4 + i] = ptr[i];
      } else if (vec == 4 && k < k_end && col + 3 < col_end) {
        const float4 t = *reinterpret_cast<const float4*>(ptr);
        reg[p * 4 + 0] = t.x; reg[p * 4 + 1] = t.y; reg[p * 4 + 2] = t.z; reg[p * 4 + 3] = t.w;
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) reg[p * 4 + i] = (k < k_end && col + i < col_end) ? ptr[i] : 0.f;
      }
    }
  }
  __device__ static inline void store(uint16_t (*S)[R][kPieceLd], const float (&reg)[kRegs]) {
    const int kg = threadIdx.x % 8, cq = threadIdx.x / 8;
    if (kUsed < kThreads && threadIdx.x >= kUsed) return;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      store_pieces<R>(S, 4 * cq + i, 4 * kg, reg[0 * 4 + i], reg[1 * 4 + i], reg[2 * 4 + i], reg[3 * 4 + i]);
  }
};

// BM x BN tile of C by 2 x 2 wavefronts, k-steps of 32.  Both operand tiles sit in LDS as three
// planes of bfloat16 pieces, [row or column][k] with k contiguous: lane l of a 32x32x16 matrix
// instruction feeds row (column) l % 32 with the eight k that start at 8 * (l / 32), one 16-byte
// read.  A and B use the same k numbering, so the product does not depend on it.  Two workgroups
// share a CU (60 KB of LDS, at most 256 registers each).
// kFast: as for the fp32 kernel.
template <int BM, int BN, bool TA, bool TB, bool kFast>
__global__ __launch_bounds__(kThreads, 2) void gemm_pieces(int64_t m_base, int64_t M, int64_t N, int64_t K,
                                                            const float* __restrict__ A, int64_t lda,
                                                            const float* __restrict__ B, int64_t ldb,
                                                            float* __restrict__ C, int64_t ldc, float beta,
                                                            int epi, int64_t k_per_split,
                                                            float* __restrict__ partial, int vecA, int vecB) {
  constexpr int BK = kPieceBK, WN = 2;
  constexpr int TM = BM / 2 / 32, TN = BN / WN / 32;
  static_assert(TM >= 1 && TN >= 1, "wave tile must hold at least one 32x32 MFMA tile");
  using LoadA = typename std::conditional<TA, MContigK4<BM>, KContig<BM, BK>>::type;
  using LoadB = typename std::conditional<TB, KContig<BN, BK>, MContigK4<BN>>::type;

  __shared__ __attribute__((aligned(16))) uint16_t As[3][BM][kPieceLd];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[3][BN][kPieceLd];

  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // a scalar
  const int wm = wave / WN, wn = wave % WN;
  int64_t tile_m, tile_n, split;
  if (!decode_tile(M - m_base, N, K, BM, BN, k_per_split, &tile_m, &tile_n, &split)) return;
  const int64_t m0 = m_base + tile_m * BM;
  const int64_t n0 = tile_n * BN;
  const int64_t kb = split * k_per_split;
  const int64_t ke = min(K, kb + k_per_split);

  float16v acc[TM][TN], fine[TM][TN];  // products of the two upper pieces; all smaller products
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = fine[i][j][r] = 0.f;

  float ra[LoadA::kRegs], rb[LoadB::kRegs];
#pragma unroll
  for (int i = 0; i < LoadA::kRegs; ++i) ra[i] = 0.f;
#pragma unroll
  for (int i = 0; i < LoadB::kRegs; ++i) rb[i] = 0.f;
  const bool whole = kFast && m0 + BM <= M;  // uniform over the block
  auto load_step = [&](int64_t k) {
    if (whole && k + BK <= ke) {
      LoadA::template load<true>(A, lda, m0, M, k, ke, 4, ra);
      LoadB::template load<true>(B, ldb, n0, N, k, ke, 4, rb);
    } else {
      LoadA::template load<false>(A, lda, m0, M, k, ke, vecA, ra);
      LoadB::template load<false>(B, ldb, n0, N, k, ke, vecB, rb);
    }
  };
  load_step(kb);

  const int frow = lane >> 5, fcol = lane & 31;
  for (int64_t k0 = kb; k0 < ke; k0 += BK) {
    if constexpr (TA) LoadA::store(As, ra); else store_pieces_kcontig<BM>(As, ra);
    if constexpr (TB) store_pieces_kcontig<BN>(Bs, rb); else LoadB::store(Bs, rb);
    __syncthreads();
    if (k0 + BK < ke) load_step(k0 + BK);  // in flight during the matrix instructions below
#pragma unroll
    for (int ks = 0; ks < BK; ks += 16) {
      bf16x8 a[TM][3], b[TN][3];
#pragma unroll
      for (int pl = 0; pl < 3; ++pl) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
          a[i][pl] = *reinterpret_cast<const bf16x8*>(&As[pl][(wm * TM + i) * 32 + fcol][ks + 8 * frow]);
#pragma unroll
        for (int j = 0; j < TN; ++j)
          b[j][pl] = *reinterpret_cast<const bf16x8*>(&Bs[pl][(wn * TN + j) * 32 + fcol][ks + 8 * frow]);
      }
      // (piece of a, piece of b), smallest products first; consecutive instructions go to
      // different accumulators.  The five small products have an accumulator of their own: the
      // matrix unit cuts an addend off below the accumulator's last bits instead of rounding it,
      // and next to the large sum that bias of the small terms would add up over a long K
      // (measured on positive operands: -2e-5 relative at K = 16384 in one accumulator, none in two).
      constexpr int kOrder[5][2] = {{2, 0}, {0, 2}, {1, 1}, {1, 0}, {0, 1}};
#pragma unroll
      for (int o = 0; o < 5; ++o)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            fine[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i][kOrder[o][0]], b[j][kOrder[o][1]], fine[i][j], 0, 0, 0);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i][0], b[j][0], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] += fine[i][j][r];
  write_tiles<TM, TN>(acc, m0 + wm * TM * 32, n0 + wn * TN * 32, M, N, split, C, ldc, beta, epi, partial);
}

// Sum of the split-K partial products, in a fixed order: 8 lanes share one output element, each
// adds every 8th split, then the 8 are folded by a shuffle tree.
__global__ __launch_bounds__(kThreads) void gemm_reduce_splits(int64_t M, int64_t N, int splits,
                                                                const float* __restrict__ partial,
                                                                float* __restrict__ C, int64_t ldc,
                                                                float beta, int epi) {
  constexpr int ZL = 8;
  const int zl = threadIdx.x % ZL;
  const int64_t idx = ((int64_t)blockIdx.x * kThreads + threadIdx.x) / ZL;
  const bool live = idx < M * N;
  float s = 0.f;
  if (live)
    for (int z = zl; z < splits; z += ZL) s += partial[(int64_t)z * M * N + idx];
#pragma unroll
  for (int d = 1; d < ZL; d <<= 1) s += __shfl_xor(s, d);
  if (live && zl == 0) {
    float* dst = C + (idx / N) * ldc + (idx % N);
    const float old = (beta != 0.f || epi == MGGCN_EPI_RELU_MASK) ? *dst : 0.f;
    *dst = gemm_epilogue(s, old, beta, epi);
  }
}

struct Shape {
  bool pieces;  // the bfloat16-piece kernel (128 x bn tiles, k-steps of 32) instead of the fp32 one
  bool wide;    // the fp32 kernel with 128 x 128 tiles (gemm_stream; aligned operands, N a multiple of 128)
  int bn, bk;
  int64_t tiles_m, tiles_n;
  int splits;
  int64_t k_per_split;
};

// per-lane byte offsets of a 128-row tile stay below 2^31 for rows shorter than this
constexpr int64_t kStreamMaxLd = (int64_t)1 << 21;
constexpr int kBM = 128, kBN = 64;  // fp32 kernel: 72 VGPRs + 32 accumulators, 4 wavefronts per SIMD

// pieces: the caller asked for the bfloat16-piece kernel (it needs two k-steps of 32 to pay);
// aligned: rows of both operands start on 16-byte boundaries
Shape plan_shape(bool pieces, bool aligned, int opA, int64_t M, int64_t N, int64_t K) {
  Shape s;
  s.pieces = pieces && K >= 64;
  s.bk = (K >= 64) ? 32 : 16;
  s.wide = !s.pieces && aligned && s.bk == 32 && N % 128 == 0;
  s.bn = s.pieces ? (N > 64 ? 128 : 64) : (s.wide ? 128 : kBN);
  const int BK = s.bk;
  s.tiles_m = ceil_div(std::max<int64_t>(M, 1), kBM);
  s.tiles_n = ceil_div(std::max<int64_t>(N, 1), s.bn);
  s.splits = 1;
  s.k_per_split = std::max<int64_t>(align_up((size_t)std::max<int64_t>(K, 1), BK), BK);
  if (opA == MGGCN_OP_T && K > 4096) {
    const int64_t tiles = s.tiles_m * s.tiles_n;
    // all workgroups resident at once: 256 CUs x 4, or x 2 for the kernels with 128 x 128 tiles and
    // their 60-67 KB of LDS (a few more would run as a second round behind the first and double
    // the kernel's time)
    // (gemm_stream with 128 x 64 tiles: 50-55 KB of LDS, three per CU)
    const bool narrow_stream = !s.pieces && !s.wide && aligned && s.bk == 32 && N % kBN == 0;
    int64_t want = std::max<int64_t>((s.pieces || s.wide ? 512 : narrow_stream ? 768 : 1024) / tiles, 1);
    want = std::min<int64_t>(want, ceil_div(K, 16 * BK));
    want = std::max<int64_t>(want, 1);
    s.k_per_split = (int64_t)align_up((size_t)ceil_div(K, want), BK);
    s.splits = (int)ceil_div(K, s.k_per_split);
  }
  return s;
}

struct GemmArgs {
  int opA, opB;
  int64_t M, N, K;
  const float* A;
  int64_t lda;
  const float* B;
  int64_t ldb;
  float* C;
  int64_t ldc;
  float beta;
  int epi;
  float* partial;
  int vecA, vecB;
  hipStream_t st;
};

#define MGGCN_GEMM_ARGS \
  0, g.M, g.N, g.K, g.A, g.lda, g.B, g.ldb, g.C, g.ldc, g.beta, g.epi, s.k_per_split, g.partial, g.vecA, g.vecB

template <int BK, bool kFast>
void launch_fp32(const GemmArgs& g, const Shape& s, dim3 grid) {
#define MGGCN_GEMM_LAUNCH(TA, TB) gemm_mfma<kBM, kBN, BK, 4, 1, TA, TB, kFast><<<grid, kThreads, 0, g.st>>>(MGGCN_GEMM_ARGS)
  if (g.opA == MGGCN_OP_N && g.opB == MGGCN_OP_N) MGGCN_GEMM_LAUNCH(false, false);
  else if (g.opA == MGGCN_OP_T && g.opB == MGGCN_OP_N) MGGCN_GEMM_LAUNCH(true, false);
  else if (g.opA == MGGCN_OP_N && g.opB == MGGCN_OP_T) MGGCN_GEMM_LAUNCH(false, true);
  else MGGCN_GEMM_LAUNCH(true, true);
#undef MGGCN_GEMM_LAUNCH
}

template <int BN, bool kFast>
void launch_pieces(const GemmArgs& g, const Shape& s, dim3 grid) {
#define MGGCN_GEMM_LAUNCH(TA, TB) gemm_pieces<kBM, BN, TA, TB, kFast><<<grid, kThreads, 0, g.st>>>(MGGCN_GEMM_ARGS)
  if (g.opA == MGGCN_OP_N && g.opB == MGGCN_OP_N) MGGCN_GEMM_LAUNCH(false, false);
  else if (g.opA == MGGCN_OP_T && g.opB == MGGCN_OP_N) MGGCN_GEMM_LAUNCH(true, false);
  else if (g.opA == MGGCN_OP_N && g.opB == MGGCN_OP_T) MGGCN_GEMM_LAUNCH(false, true);
  else MGGCN_GEMM_LAUNCH(true, true);
#undef MGGCN_GEMM_LAUNCH
}
#undef MGGCN_GEMM_ARGS

int launch_all(const GemmArgs& g, const Shape& s) {
  // unsplit: whole groups of 8 M tiles (one per XCD), the kernel drops the padding
  const int64_t nblk = s.splits == 1 ? kXcds * ceil_div(s.tiles_m, kXcds) * s.tiles_n
                                     : (int64_t)s.splits * s.tiles_m * s.tiles_n;
  MGGCN_REQUIRE(nblk < ((int64_t)1 << 31), MGGCN_E_OVERFLOW, "GeMM grid of %lld x %lld x %d tiles too large",
                (long long)s.tiles_m, (long long)s.tiles_n, s.splits);
  const dim3 grid((unsigned)nblk, 1, 1);
  // whole tiles along N and 16-byte rows: interior blocks load without any check
  const bool fast = g.vecA == 4 && g.vecB == 4 && g.N % s.bn == 0;
  if (s.pieces) {
    if (s.bn == 128) fast ? launch_pieces<128, true>(g, s, grid) : launch_pieces<128, false>(g, s, grid);
    else fast ? launch_pieces<64, true>(g, s, grid) : launch_pieces<64, false>(g, s, grid);
  } else if (s.bk == 32 && fast && g.lda < kStreamMaxLd && g.ldb < kStreamMaxLd) {
    // as many workgroups as the chip holds at once (a multiple of 8); each walks its share of the tiles
    const dim3 pgrid((unsigned)std::min<int64_t>(nblk, (s.wide ? 2 : 3) * 256), 1, 1);
#define MGGCN_GEMM_LAUNCH(TA, TB)                                                                               \
  do {                                                                                                          \
    if (s.wide)                                                                                                 \
      gemm_stream<128, 2, 2, TA, TB><<<pgrid, kThreads, 0, g.st>>>(g.M, g.N, g.K, g.A, g.lda, g.B, g.ldb, g.C, g.ldc, \
                                                                   g.beta, g.epi, s.k_per_split, g.partial,       \
                                                                   (uint32_t)nblk, (uint32_t)s.tiles_m,           \
                                                                   (uint32_t)s.tiles_n, (uint32_t)s.splits);      \
    else                                                                                                        \
      gemm_stream<64, 4, 1, TA, TB><<<pgrid, kThreads, 0, g.st>>>(g.M, g.N, g.K, g.A, g.lda, g.B, g.ldb, g.C, g.ldc,  \
                                                                  g.beta, g.epi, s.k_per_split, g.partial,        \
                                                                  (uint32_t)nblk, (uint32_t)s.tiles_m,            \
                                                                  (uint32_t)s.tiles_n, (uint32_t)s.splits);       \
  } while (0)
    if (g.opA == MGGCN_OP_N && g.opB == MGGCN_OP_N) MGGCN_GEMM_LAUNCH(false, false);
    else if (g.opA == MGGCN_OP_T && g.opB == MGGCN_OP_N) MGGCN_GEMM_LAUNCH(true, false);
    else if (g.opA == MGGCN_OP_N && g.opB == MGGCN_OP_T) MGGCN_GEMM_LAUNCH(false, true);
    else MGGCN_GEMM_LAUNCH(true, true);
#undef MGGCN_GEMM_LAUNCH
  } else if (s.bk == 32) {
    fast ? launch_fp32<32, true>(g, s, grid) : launch_fp32<32, false>(g, s, grid);
  } else {
    fast ? launch_fp32<16, true>(g, s, grid) : launch_fp32<16, false>(g, s, grid);
  }
  MGGCN_LAUNCH_CHECK();
  return MGGCN_OK;
}

}  // namespace

int gemm_run(bool pieces, int opA, int opB, int64_t M, int64_t N, int64_t K, const float* A, int64_t lda,
             const float* B, int64_t ldb, float beta, int epilogue, float* C, int64_t ldc, void* ws,
             size_t ws_bytes, void* stream) {
  MGGCN_REQUIRE((opA == MGGCN_OP_N || opA == MGGCN_OP_T) && (opB == MGGCN_OP_N || opB == MGGCN_OP_T),
                MGGCN_E_INVALID_ARG, "unknown op (%d, %d)", opA, opB);
  MGGCN_REQUIRE(M >= 0 && N >= 0 && K >= 0, MGGCN_E_INVALID_ARG, "negative size M=%lld N=%lld K=%lld",
                (long long)M, (long long)N, (long long)K);
  MGGCN_REQUIRE(beta == 0.f || beta == 1.f, MGGCN_E_INVALID_ARG, "beta must be 0 or 1");
  MGGCN_REQUIRE(epilogue == MGGCN_EPI_NONE || epilogue == MGGCN_EPI_RELU || epilogue == MGGCN_EPI_RELU_MASK,
                MGGCN_E_INVALID_ARG, "unknown epilogue %d", epilogue);
  MGGCN_REQUIRE(!(epilogue == MGGCN_EPI_RELU_MASK && beta != 0.f), MGGCN_E_INVALID_ARG,
                "RELU_MASK cannot be combined with beta = 1");
  const int64_t a_cols = (opA == MGGCN_OP_N) ? K : M, b_cols = (opB == MGGCN_OP_N) ? N : K;
  MGGCN_REQUIRE(lda >= a_cols && ldb >= b_cols && ldc >= N, MGGCN_E_INVALID_ARG,
                "leading dimension too small (lda %lld/%lld, ldb %lld/%lld, ldc %lld/%lld)",
                (long long)lda, (long long)a_cols, (long long)ldb, (long long)b_cols, (long long)ldc,
                (long long)N);
  if (M == 0 || N == 0) return MGGCN_OK;
  MGGCN_REQUIRE(C != nullptr, MGGCN_E_INVALID_ARG, "C is NULL");
  MGGCN_REQUIRE(K == 0 || (A && B), MGGCN_E_INVALID_ARG, "A / B is NULL");
  auto vec_width = [](const float* p, int64_t ld) {
    if (aligned(p, 16) && ld % 4 == 0) return 4;
    if (aligned(p, 8) && ld % 2 == 0) return 2;
    return 1;
  };
  const int vecA = vec_width(A, lda), vecB = vec_width(B, ldb);
  const bool rows16 = vecA == 4 && vecB == 4 && lda < kStreamMaxLd && ldb < kStreamMaxLd;
  const Shape s = plan_shape(pieces, rows16, opA, M, N, std::max<int64_t>(K, 1));
  float* partial = nullptr;
  if (s.splits > 1) {
    const size_t need = mggcn_gemm_workspace_bytes(opA, opB, M, N, K);  // one size for both kernels
    MGGCN_REQUIRE(ws && aligned(ws, kWsAlign), MGGCN_E_WORKSPACE, "workspace is NULL or not 256-byte aligned");
    MGGCN_REQUIRE(ws_bytes >= need, MGGCN_E_WORKSPACE, "workspace too small: %zu bytes given, %zu needed",
                  ws_bytes, need);
    partial = static_cast<float*>(ws);
  }
  GemmArgs g{opA, opB, M, N, K, A, lda, B, ldb, C, ldc, beta, epilogue, partial, vecA, vecB, as_stream(stream)};
  hipStream_t st = g.st;
  const int rc = launch_all(g, s);
  if (rc) return rc;
  if (partial) {
    gemm_reduce_splits<<<(unsigned)ceil_div(M * N * 8, kThreads), kThreads, 0, st>>>(M, N, s.splits, partial,
                                                                                    C, ldc, beta, epilogue);
    MGGCN_LAUNCH_CHECK();
  }
  return MGGCN_OK;
}

}  // namespace mggcn

using namespace mggcn;

extern "C" {

size_t mggcn_gemm_workspace_bytes(int opA, int opB, int64_t M, int64_t N, int64_t K) {
  (void)opB;
  if (M <= 0 || N <= 0 || K <= 0) return 0;
  // enough for every kernel: they cut the inner dimension into different numbers of parts
  const int splits = std::max({plan_shape(false, false, opA, M, N, K).splits, plan_shape(false, true, opA, M, N, K).splits,
                               plan_shape(true, false, opA, M, N, K).splits});
  if (splits <= 1) return 0;
  return align_up((size_t)splits * (size_t)M * (size_t)N * sizeof(float), kWsAlign);
}

int mggcn_gemm(int opA, int opB, int64_t M, int64_t N, int64_t K, const float* A, int64_t lda,
               const float* B, int64_t ldb, float beta, int epilogue, float* C, int64_t ldc, void* ws,
               size_t ws_bytes, void* stream) {
  return gemm_run(false, opA, opB, M, N, K, A, lda, B, ldb, beta, epilogue, C, ldc, ws, ws_bytes, stream);
}

int mggcn_gemm_bf16x3(int opA, int opB, int64_t M, int64_t N, int64_t K, const float* A, int64_t lda,
                      const float* B, int64_t ldb, float beta, int epilogue, float* C, int64_t ldc, void* ws,
                      size_t ws_bytes, void* stream) {
  return gemm_run(true, opA, opB, M, N, K, A, lda, B, ldb, beta, epilogue, C, ldc, ws, ws_bytes, stream);
}

}  // extern "C"
