// Dense fp32 GeMM on the CDNA matrix cores for the three products of a GCN layer
// (Eq. 5: H W, Eq. 10: H^T HW_G, Eq. 11: HW_G W^T of the paper).
//
//   C = epilogue( op(A) op(B) + beta C )
//
// One kernel template.  A workgroup of 4 wavefronts owns a BM x BN tile of C and walks K in
// steps of 32 (16 for a short inner dimension).  Both operand tiles are staged through LDS in k-major order (As[k][m], Bs[k][n])
// whatever their layout in memory, because that is the order v_mfma_f32_32x32x2_f32 wants its
// fragments in: lane l feeds A[m = l%32][k = l/32] and B[k = l/32][n = l%32], so a fragment is
// 32 consecutive floats of one LDS row and is read without bank conflicts.  The next k-step's
// global loads are issued before the MFMA loop of the current one.
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
};

__device__ inline float gemm_epilogue(float acc, float old, float beta, int epi) {
  if (beta != 0.f) acc += old;
  if (epi == MGGCN_EPI_RELU) acc = acc > 0.f ? acc : 0.f;
  if (epi == MGGCN_EPI_RELU_MASK) acc = old > 0.f ? acc : 0.f;
  return acc;
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

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / WN, wn = wave % WN;
  // Workgroups are dealt to the 8 XCDs round-robin by index, and each XCD has its own L2.  The
  // 1-D grid is therefore decoded so that the N tiles of one M tile -- they re-read the same rows
  // of A -- sit on one XCD next to each other in time.  Measured on 2.45M x 256 x 256: 3.33 ->
  // 2.91 ms, A being fetched from HBM once instead of four times.  With a split inner dimension
  // the tiles of a split read disjoint columns of A, and the plain order (M tiles fastest, spread
  // over the XCDs) measured faster than grouping a split on one XCD.
  const int64_t tiles_m = (M - m_base + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  const int64_t splits = (K + k_per_split - 1) / k_per_split;
  int64_t tile_m, tile_n, split;
  if (splits == 1) {
    const int64_t xcd = blockIdx.x % kXcds, local = blockIdx.x / kXcds;
    tile_n = local % tiles_n;
    tile_m = (local / tiles_n) * kXcds + xcd;
    split = 0;
    if (tile_m >= tiles_m) return;  // padding of the grid to whole groups of 8
  } else {
    const int64_t per = tiles_m * tiles_n, t = blockIdx.x % per;
    split = blockIdx.x / per;
    tile_m = t % tiles_m;
    tile_n = t / tiles_m;
  }
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

  // accumulator register r of lane l is C[8*(r/4) + 4*(l/32) + r%4][l%32] of its 32x32 tile
  const bool to_partial = partial != nullptr;
  float* out = to_partial ? partial + split * M * N : C;
  const int64_t ldo = to_partial ? N : ldc;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int64_t col = n0 + (wn * TN + j) * 32 + fcol;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t row = m0 + (wm * TM + i) * 32 + 8 * (r / 4) + 4 * frow + (r % 4);
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
  int bk;
  int64_t tiles_m, tiles_n;
  int splits;
  int64_t k_per_split;
};

constexpr int kBM = 128, kBN = 64;  // 72 VGPRs + 32 accumulators: 4 wavefronts per SIMD

Shape plan_shape(int opA, int64_t M, int64_t N, int64_t K) {
  Shape s;
  s.bk = (K >= 64) ? 32 : 16;
  const int BK = s.bk;
  s.tiles_m = ceil_div(std::max<int64_t>(M, 1), kBM);
  s.tiles_n = ceil_div(std::max<int64_t>(N, 1), kBN);
  s.splits = 1;
  s.k_per_split = std::max<int64_t>(align_up((size_t)std::max<int64_t>(K, 1), BK), BK);
  if (opA == MGGCN_OP_T && K > 4096) {
    const int64_t tiles = s.tiles_m * s.tiles_n;
    // all workgroups resident at once: 256 CUs x 4 (a few more would run as a second round
    // behind the first and double the kernel's time)
    int64_t want = std::max<int64_t>(1024 / tiles, 1);
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

template <int BK, bool kFast>
int launch_rows(const GemmArgs& g, const Shape& s, int64_t m_base, int64_t m_tiles) {
  if (m_tiles <= 0) return MGGCN_OK;
  // unsplit: whole groups of 8 M tiles (one per XCD), the kernel drops the padding
  const int64_t nblk = s.splits == 1 ? kXcds * ceil_div(m_tiles, kXcds) * s.tiles_n
                                     : (int64_t)s.splits * m_tiles * s.tiles_n;
  MGGCN_REQUIRE(nblk < ((int64_t)1 << 31), MGGCN_E_OVERFLOW, "GeMM grid of %lld x %lld x %d tiles too large",
                (long long)m_tiles, (long long)s.tiles_n, s.splits);
  dim3 grid((unsigned)nblk, 1, 1);
#define MGGCN_GEMM_LAUNCH(TA, TB)                                                                              \
  gemm_mfma<kBM, kBN, BK, 4, 1, TA, TB, kFast><<<grid, kThreads, 0, g.st>>>(                                   \
      m_base, g.M, g.N, g.K, g.A, g.lda, g.B, g.ldb, g.C, g.ldc, g.beta, g.epi, s.k_per_split, g.partial, g.vecA, \
      g.vecB)
  if (g.opA == MGGCN_OP_N && g.opB == MGGCN_OP_N) MGGCN_GEMM_LAUNCH(false, false);
  else if (g.opA == MGGCN_OP_T && g.opB == MGGCN_OP_N) MGGCN_GEMM_LAUNCH(true, false);
  else if (g.opA == MGGCN_OP_N && g.opB == MGGCN_OP_T) MGGCN_GEMM_LAUNCH(false, true);
  else MGGCN_GEMM_LAUNCH(true, true);
#undef MGGCN_GEMM_LAUNCH
  MGGCN_LAUNCH_CHECK();
  return MGGCN_OK;
}

template <int BK>
int launch_all(const GemmArgs& g, const Shape& s) {
  const bool fast_ok = g.vecA == 4 && g.vecB == 4 && g.N % kBN == 0;
  return fast_ok ? launch_rows<BK, true>(g, s, 0, s.tiles_m) : launch_rows<BK, false>(g, s, 0, s.tiles_m);
}

}  // namespace
}  // namespace mggcn

using namespace mggcn;

extern "C" {

size_t mggcn_gemm_workspace_bytes(int opA, int opB, int64_t M, int64_t N, int64_t K) {
  (void)opB;
  if (M <= 0 || N <= 0 || K <= 0) return 0;
  const Shape s = plan_shape(opA, M, N, K);
  if (s.splits <= 1) return 0;
  return align_up((size_t)s.splits * (size_t)M * (size_t)N * sizeof(float), kWsAlign);
}

int mggcn_gemm(int opA, int opB, int64_t M, int64_t N, int64_t K, const float* A, int64_t lda,
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
  const Shape s = plan_shape(opA, M, N, std::max<int64_t>(K, 1));
  float* partial = nullptr;
  if (s.splits > 1) {
    const size_t need = mggcn_gemm_workspace_bytes(opA, opB, M, N, K);
    MGGCN_REQUIRE(ws && aligned(ws, kWsAlign), MGGCN_E_WORKSPACE, "workspace is NULL or not 256-byte aligned");
    MGGCN_REQUIRE(ws_bytes >= need, MGGCN_E_WORKSPACE, "workspace too small: %zu bytes given, %zu needed",
                  ws_bytes, need);
    partial = static_cast<float*>(ws);
  }
  auto vec_width = [](const float* p, int64_t ld) {
    if (aligned(p, 16) && ld % 4 == 0) return 4;
    if (aligned(p, 8) && ld % 2 == 0) return 2;
    return 1;
  };
  GemmArgs g{opA, opB, M, N, K, A, lda, B, ldb, C, ldc, beta, epilogue, partial, vec_width(A, lda), vec_width(B, ldb),
             as_stream(stream)};
  hipStream_t st = g.st;
  const int rc = (s.bk == 32) ? launch_all<32>(g, s) : launch_all<16>(g, s);
  if (rc) return rc;
  if (partial) {
    gemm_reduce_splits<<<(unsigned)ceil_div(M * N * 8, kThreads), kThreads, 0, st>>>(M, N, s.splits, partial,
                                                                                    C, ldc, beta, epilogue);
    MGGCN_LAUNCH_CHECK();
  }
  return MGGCN_OK;
}

}  // extern "C"
