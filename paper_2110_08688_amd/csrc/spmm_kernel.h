// The row-segment SpMM kernel and its launch dispatch, generic over the element type of the
// gathered operand (fp32, or a bfloat16 copy that halves the gather traffic; accumulation and
// output are fp32 either way).  Included by one translation unit per element type.
#pragma once

#include "common.h"
#include "graph.h"
#include "spmm_device.h"

namespace mggcn {

constexpr int kSpmmThreads = 256;

struct bf16_t { uint16_t bits; };  // bfloat16 storage: the upper half of an fp32

// How a lane holds and consumes VW consecutive elements of a gathered row.
template <typename XT, int VW>
struct Operand;

template <int VW>
struct Operand<float, VW> {
  struct Raw { float v[VW]; };
  __device__ static inline void zero(Raw& r) {
#pragma unroll
    for (int i = 0; i < VW; ++i) r.v[i] = 0.f;
  }
  __device__ static inline void load(const char* __restrict__ p, Raw& r) {
    load_vec<VW>(reinterpret_cast<const float*>(p), r.v);
  }
  __device__ static inline void fma(float a, const Raw& r, float (&acc)[VW]) {
#pragma unroll
    for (int i = 0; i < VW; ++i) acc[i] = fmaf(a, r.v[i], acc[i]);
  }
};

// Eight bfloat16 = one 16-byte load, kept packed while in flight (4 registers, as many as the
// fp32 path spends on 4 elements) and widened on use: an element is the upper half of an fp32.
template <>
struct Operand<bf16_t, 8> {
  struct Raw { uint32_t w[4]; };
  __device__ static inline void zero(Raw& r) { r.w[0] = r.w[1] = r.w[2] = r.w[3] = 0u; }
  __device__ static inline void load(const char* __restrict__ p, Raw& r) {
    const uint4 t = *reinterpret_cast<const uint4*>(p);
    r.w[0] = t.x; r.w[1] = t.y; r.w[2] = t.z; r.w[3] = t.w;
  }
  __device__ static inline void fma(float a, const Raw& r, float (&acc)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      acc[2 * i] = fmaf(a, __uint_as_float(r.w[i] << 16), acc[2 * i]);
      acc[2 * i + 1] = fmaf(a, __uint_as_float(r.w[i] & 0xFFFF0000u), acc[2 * i + 1]);
    }
  }
};

template <>
struct Operand<bf16_t, 1> {
  struct Raw { float v; };
  __device__ static inline void zero(Raw& r) { r.v = 0.f; }
  __device__ static inline void load(const char* __restrict__ p, Raw& r) {
    r.v = __uint_as_float((uint32_t)*reinterpret_cast<const uint16_t*>(p) << 16);
  }
  __device__ static inline void fma(float a, const Raw& r, float (&acc)[1]) { acc[0] = fmaf(a, r.v, acc[0]); }
};

// One workgroup's share of one length bin: `tb` is the workgroup's index inside the bin, `chunk`
// its feature chunk.
template <typename XT, int VW, int LPR, int GPT, int UMAX>
__device__ __forceinline__ void spmm_team_body(
    int64_t tb, int chunk, const Task* __restrict__ tasks, int64_t ntasks, const int32_t* __restrict__ colidx,
    const float* __restrict__ val, const XT* __restrict__ X, uint32_t ldx_bytes, int F,
    float beta, int epi, float* __restrict__ Y, int64_t ldy, float* __restrict__ partial,
    int64_t ldp) {
  constexpr int TEAM = LPR * GPT;
  constexpr int TPW = 64 / TEAM;
  constexpr int U = LPR < UMAX ? LPR : UMAX;
  static_assert(TEAM <= 64 && TPW >= 1, "team must fit a wavefront");

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int team = lane / TEAM, tl = lane % TEAM;
  const int g = tl / LPR, fl = tl % LPR;
  const int team_base = team * TEAM;
  const int64_t t = (tb * (kSpmmThreads / 64) + wave) * TPW + team;

  Task task = {0, 0u, 0u, -1};
  const bool has_task = t < ntasks;
  if (has_task) task = tasks[t];
  const int len = (int)(task.len_flags & kTaskLenMask);

  // longest and shortest task of this wavefront: uniform loop bounds, so the shuffles below
  // are executed by all lanes together
  int maxlen = len, minlen = len;
#pragma unroll
  for (int d = TEAM; d < 64; d <<= 1) {
    maxlen = max(maxlen, __shfl_xor(maxlen, d));
    minlen = min(minlen, __shfl_xor(minlen, d));
  }
  maxlen = __builtin_amdgcn_readfirstlane(maxlen);
  minlen = __builtin_amdgcn_readfirstlane(minlen);

  const int f0 = chunk * (LPR * VW) + fl * VW;
  const int nf = min(VW, max(0, F - f0));
  const bool live = nf > 0;  // this lane covers at least one feature column
  const char* __restrict__ xbase = reinterpret_cast<const char*>(X + f0);
  const int32_t* __restrict__ cptr = colidx + ((size_t)task.k0 + tl);
  const float* __restrict__ vptr = val + ((size_t)task.k0 + tl);

  using Op = Operand<XT, VW>;
  float acc[VW];
  typename Op::Raw xs[U];
#pragma unroll
  for (int i = 0; i < VW; ++i) acc[i] = 0.f;
#pragma unroll
  for (int u = 0; u < U; ++u) Op::zero(xs[u]);

  int c = 0;
  float v = 0.f;
  if (tl < len) {
    c = __builtin_nontemporal_load(cptr);
    v = __builtin_nontemporal_load(vptr);
  }
  // what the output row holds now, if the epilogue needs it: fetched up front so that its
  // latency hides behind the gathers
  const float my_beta = (task.len_flags & kTaskFirst) ? beta : 1.f;
  const int my_epi = (task.len_flags & kTaskLast) ? epi : (int)MGGCN_EPI_NONE;
  const bool to_y = has_task && g == 0 && live && task.slot < 0;
  float old[VW];
#pragma unroll
  for (int i = 0; i < VW; ++i) old[i] = 0.f;
  if (to_y && (my_beta != 0.f || my_epi == MGGCN_EPI_RELU_MASK)) load_row<VW>(Y + (int64_t)task.row * ldy + f0, nf, old);
  for (int base = 0; base < maxlen; base += TEAM) {
    int c_next = 0;
    float v_next = 0.f;
    if (base + TEAM + tl < len) {
      c_next = __builtin_nontemporal_load(cptr + base + TEAM);
      v_next = __builtin_nontemporal_load(vptr + base + TEAM);
    }
    // full step: every team of the wavefront still has TEAM entries, nothing to predicate
    const bool full = base + TEAM <= minlen;
    const int remaining = maxlen - base;  // uniform
#pragma unroll 1
    for (int j0 = 0; j0 < LPR; j0 += U) {
      if (j0 * GPT >= remaining) break;
      int cj[U];
      float vs[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int src = team_base + (j0 + u) * GPT + g;  // entry handled by my lane group
        cj[u] = __shfl(c, src);
        vs[u] = __shfl(v, src);  // 0 beyond the task's end
      }
      if (full) {
        if (live) {
#pragma unroll
          for (int u = 0; u < U; ++u)
            Op::load(xbase + (uint64_t)(uint32_t)cj[u] * ldx_bytes, xs[u]);
        }
      } else {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          Op::zero(xs[u]);
          if (live && base + (j0 + u) * GPT + g < len)
            Op::load(xbase + (uint64_t)(uint32_t)cj[u] * ldx_bytes, xs[u]);
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) Op::fma(vs[u], xs[u], acc);
    }
    c = c_next;
    v = v_next;
  }

  // fold the GPT lane groups of the team
#pragma unroll
  for (int d = LPR; d < TEAM; d <<= 1)
#pragma unroll
    for (int i = 0; i < VW; ++i) acc[i] += __shfl_xor(acc[i], d);

  if (has_task && g == 0 && live) {
    if (task.slot >= 0)
      store_out<VW>(partial + (int64_t)task.slot * ldp + f0, nf, acc, 0.f, MGGCN_EPI_NONE, false);
    else {
      float r[VW];
#pragma unroll
      for (int i = 0; i < VW; ++i) r[i] = apply_epilogue(acc[i], old[i], my_beta, my_epi);
      store_out<VW>(Y + (int64_t)task.row * ldy + f0, nf, r, 0.f, MGGCN_EPI_NONE, false, (task.len_flags & kTaskLast) != 0);
    }
  }
}

// The length bins of one pass in one launch.  Tasks are sorted longest first, so a bin (tasks of
// length >= 8 << i get 1 << i lane groups) is a contiguous range of the task list; workgroups are
// numbered bin after bin, longest tasks first, and each finds its bin from the workgroup counts.
// One launch instead of one per bin lets the short tasks fill the tail of the long ones.
constexpr int kMaxBins = 7;
struct BinTable {
  int n_bins;
  int gpt_log2[kMaxBins];
  int64_t block_begin[kMaxBins + 1];  // in workgroups, feature chunks included
  int64_t task_begin[kMaxBins + 1];   // offsets into the pass's task list
};

template <typename XT, int VW, int LPR, int UMAX>
__global__ __launch_bounds__(kSpmmThreads) void spmm_tasks(
    BinTable bins, const Task* __restrict__ tasks, const int32_t* __restrict__ colidx,
    const float* __restrict__ val, const XT* __restrict__ X, uint32_t ldx_bytes, int F, int n_chunks,
    float beta, int epi, float* __restrict__ Y, int64_t ldy, float* __restrict__ partial, int64_t ldp) {
  int b = 0;
  while (b + 1 < bins.n_bins && (int64_t)blockIdx.x >= bins.block_begin[b + 1]) ++b;
  const int64_t in_bin = (int64_t)blockIdx.x - bins.block_begin[b];
  const int chunk = (int)(in_bin % n_chunks);
  const int64_t tb = in_bin / n_chunks;
  const Task* t0 = tasks + bins.task_begin[b];
  const int64_t nt = bins.task_begin[b + 1] - bins.task_begin[b];
#define MGGCN_SPMM_BIN(G)                                                                                   \
  if constexpr (LPR * (G) <= 64) {                                                                          \
    spmm_team_body<XT, VW, LPR, (G), UMAX>(tb, chunk, t0, nt, colidx, val, X, ldx_bytes, F, beta, epi, Y, ldy, \
                                           partial, ldp);                                                   \
  }
  switch (bins.gpt_log2[b]) {  // uniform over the workgroup
    case 0: MGGCN_SPMM_BIN(1) break;
    case 1: MGGCN_SPMM_BIN(2) break;
    case 2: MGGCN_SPMM_BIN(4) break;
    case 3: MGGCN_SPMM_BIN(8) break;
    case 4: MGGCN_SPMM_BIN(16) break;
    case 5: MGGCN_SPMM_BIN(32) break;
    default: MGGCN_SPMM_BIN(64) break;
  }
#undef MGGCN_SPMM_BIN
}

struct LaunchArgs {
  BinTable bins;      // the length bins of this pass
  const Task* tasks;  // the pass's task list (device)
  const int32_t* colidx;
  const float* val;
  const void* X;  // float or bfloat16 rows
  int64_t ldx;
  int F, n_chunks;
  float beta;
  int epi;
  float* Y;
  int64_t ldy;
  float* partial;
  int64_t ldp;
  hipStream_t stream;
};

// workgroups one bin needs at `lpr` lanes per row: (1 << gpt_log2) lane groups per task
inline int64_t spmm_bin_blocks(int64_t ntasks, int lpr, int gpt_log2, int n_chunks) {
  const int64_t teams_per_block = (kSpmmThreads / 64) * (64 / (lpr << gpt_log2));
  return ceil_div(ntasks, teams_per_block) * n_chunks;
}

template <typename XT, int VW, int LPR>
int launch_one(const LaunchArgs& a) {
  const int64_t blocks = a.bins.block_begin[a.bins.n_bins];
  MGGCN_REQUIRE(blocks < ((int64_t)1 << 31), MGGCN_E_OVERFLOW, "SpMM grid of %lld blocks too large",
                (long long)blocks);
  if (blocks == 0) return MGGCN_OK;
  // 4 gathers per lane in flight: <= 64 VGPRs, 8 wavefronts per SIMD (8 in flight measured no faster)
  spmm_tasks<XT, VW, LPR, 4><<<(unsigned)blocks, kSpmmThreads, 0, a.stream>>>(
      a.bins, a.tasks, a.colidx, a.val, static_cast<const XT*>(a.X), (uint32_t)(a.ldx * (int64_t)sizeof(XT)),
      a.F, a.n_chunks, a.beta, a.epi, a.Y, a.ldy, a.partial, a.ldp);
  MGGCN_LAUNCH_CHECK();
  return MGGCN_OK;
}

template <typename XT, int VW>
int launch_lpr(int lpr, const LaunchArgs& a) {
  switch (lpr) {
    case 1: return launch_one<XT, VW, 1>(a);
    case 2: return launch_one<XT, VW, 2>(a);
    case 4: return launch_one<XT, VW, 4>(a);
    case 8: return launch_one<XT, VW, 8>(a);
    case 16: return launch_one<XT, VW, 16>(a);
    case 32: return launch_one<XT, VW, 32>(a);
    case 64: return launch_one<XT, VW, 64>(a);
    default: break;
  }
  return fail(MGGCN_E_UNSUPPORTED, "no SpMM kernel for %d lanes per row", lpr);
}

// Runs one SpMM over the graph's task tables (all column panels and feature slices, the fix-up of
// cut rows) with `launch` starting the kernel for one pass.  Shared by the fp32 and the bfloat16
// entry points; arguments are already checked.
using SpmmLaunchFn = int (*)(int vw, int lpr, const LaunchArgs& a);
int spmm_run(const mggcn_graph* g, const Orientation& o, const void* X, int64_t ldx, int elem_bytes, int vw,
             int32_t F, float beta, int epilogue, float* Y, int64_t ldy, void* stream, SpmmLaunchFn launch);
// Argument checks common to both entry points (returns a status, sets the error text).
int spmm_check_args(const mggcn_graph* g, int op, const void* X, int64_t ldx, int elem_bytes, int32_t F,
                    float beta, int epilogue, const float* Y, int64_t ldy);

}  // namespace mggcn
