// CSR SpMM  Y = epilogue( op(A^) X + beta Y )  for gfx950 -- the product that takes most of a
// GCN epoch (Eq. 6 forward, Eq. 9 backward of the paper).
//
// Work decomposition (done once per graph on the host, the graph being fixed for all epochs):
//   every row is cut into segments of at most seg_len entries; a segment is a task.  Tasks are
//   ordered longest first.  A row with one segment is written straight to Y; the segments of a
//   cut row go to a partial-sum table and a second small kernel adds them in segment order, so
//   the result never depends on timing (no floating-point atomics).
//
// Kernel mapping (wave64):
//   the feature dimension runs along lanes: LPR lanes x VW floats cover one feature chunk of a
//   dense row, so a gathered row is read with 16-byte loads that are contiguous across lanes.
//   A team of LPR*GPT lanes owns one task: GPT lane groups walk the segment's entries
//   interleaved, and their accumulators are folded with xor-shuffles at the end.  Column
//   indices and values are fetched TEAM entries at a time with one coalesced streaming load
//   and handed to the groups by ds_bpermute.  Long tasks get the whole wave (GPT = 64/LPR);
//   short ones get narrower teams so that several rows share a wave.
//   Feature chunks map to blockIdx so that, with 2, 4 or 8 chunks, one chunk always lands on the
//   same XCDs (workgroups are dealt round-robin over the 8 XCDs): each L2 then caches a
//   1/n_chunks column slice of X instead of all of it.
#include "common.h"
#include "graph.h"

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

namespace mggcn {
namespace {

constexpr int kThreads = 256;
constexpr int kDefaultSegLen = 512;

void analyse(Orientation* o, const std::vector<int32_t>& rowptr, int32_t seg_len) {
  const int32_t n = o->n_rows;
  std::vector<Task> row_order;
  row_order.reserve((size_t)n + (size_t)(o->nnz / seg_len) + 16);
  o->fix.clear();
  int64_t slots = 0;
  for (int32_t i = 0; i < n; ++i) {
    const int32_t b = rowptr[i], len = rowptr[i + 1] - b;
    if (len <= seg_len) {
      row_order.push_back({i, b, b + len, -1});
    } else {
      const int32_t nseg = (int32_t)ceil_div(len, seg_len);
      const int32_t piece = (int32_t)ceil_div(len, nseg);
      o->fix.push_back({i, (int32_t)slots, nseg, 0});
      for (int32_t s = 0; s < nseg; ++s) {
        const int32_t k0 = b + s * piece;
        const int32_t k1 = std::min(b + len, k0 + piece);
        row_order.push_back({i, k0, k1, (int32_t)slots++});
      }
    }
  }
  o->n_slots = slots;
  // counting sort by length, longest first, row order kept inside a length
  std::vector<int64_t> start((size_t)seg_len + 2, 0);
  for (const Task& t : row_order) start[(size_t)(seg_len - (t.k1 - t.k0)) + 1]++;
  for (int32_t l = 0; l <= seg_len; ++l) start[(size_t)l + 1] += start[l];
  o->tasks.resize(row_order.size());
  for (const Task& t : row_order) o->tasks[(size_t)start[(size_t)(seg_len - (t.k1 - t.k0))]++] = t;
  for (int i = 0; i < kLenClasses; ++i) {
    const int32_t thr = 8 << i;
    // tasks are sorted descending: count of length >= thr by binary search
    int64_t lo = 0, hi = (int64_t)o->tasks.size();
    while (lo < hi) {
      const int64_t mid = (lo + hi) / 2;
      if (o->tasks[(size_t)mid].k1 - o->tasks[(size_t)mid].k0 >= thr) lo = mid + 1; else hi = mid;
    }
    o->cnt_ge[i] = lo;
  }
}

// ---------------------------------------------------------------------------------------
// device code
// ---------------------------------------------------------------------------------------

template <int VW>
__device__ inline void load_row(const float* __restrict__ p, int nf, float (&x)[VW]) {
  if (nf == VW) {
    if constexpr (VW == 4) {
      const float4 t = *reinterpret_cast<const float4*>(p);
      x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
    } else if constexpr (VW == 2) {
      const float2 t = *reinterpret_cast<const float2*>(p);
      x[0] = t.x; x[1] = t.y;
    } else {
      x[0] = p[0];
    }
  } else {
#pragma unroll
    for (int i = 0; i < VW; ++i) x[i] = (i < nf) ? p[i] : 0.f;
  }
}

__device__ inline float apply_epilogue(float acc, float old, float beta, int epi) {
  if (beta != 0.f) acc += old;
  if (epi == MGGCN_EPI_RELU) acc = acc > 0.f ? acc : 0.f;
  if (epi == MGGCN_EPI_RELU_MASK) acc = old > 0.f ? acc : 0.f;
  return acc;
}

template <int VW>
__device__ inline void store_out(float* __restrict__ dst, int nf, const float (&a)[VW], float beta,
                                 int epi, bool final_row) {
  float r[VW];
  if (final_row && (beta != 0.f || epi == MGGCN_EPI_RELU_MASK)) {
    float old[VW];
    load_row<VW>(dst, nf, old);
#pragma unroll
    for (int i = 0; i < VW; ++i) r[i] = apply_epilogue(a[i], old[i], beta, epi);
  } else if (final_row) {
#pragma unroll
    for (int i = 0; i < VW; ++i) r[i] = apply_epilogue(a[i], 0.f, 0.f, epi);
  } else {
#pragma unroll
    for (int i = 0; i < VW; ++i) r[i] = a[i];
  }
  if (nf == VW) {
    if constexpr (VW == 4) {
      *reinterpret_cast<float4*>(dst) = make_float4(r[0], r[1], r[2], r[3]);
    } else if constexpr (VW == 2) {
      *reinterpret_cast<float2*>(dst) = make_float2(r[0], r[1]);
    } else {
      dst[0] = r[0];
    }
  } else {
#pragma unroll
    for (int i = 0; i < VW; ++i)
      if (i < nf) dst[i] = r[i];
  }
}

template <int VW, int LPR, int GPT>
__global__ __launch_bounds__(kThreads) void spmm_tasks(
    const Task* __restrict__ tasks, int64_t ntasks, const int32_t* __restrict__ colidx,
    const float* __restrict__ val, const float* __restrict__ X, int64_t ldx, int F, int n_chunks,
    float beta, int epi, float* __restrict__ Y, int64_t ldy, float* __restrict__ partial,
    int64_t ldp) {
  constexpr int TEAM = LPR * GPT;
  constexpr int TPW = 64 / TEAM;
  constexpr int U = LPR < 8 ? LPR : 8;
  static_assert(TEAM <= 64 && TPW >= 1, "team must fit a wavefront");

  const int chunk = (int)(blockIdx.x % (unsigned)n_chunks);
  const int64_t tb = blockIdx.x / (unsigned)n_chunks;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int team = lane / TEAM, tl = lane % TEAM;
  const int g = tl / LPR, fl = tl % LPR;
  const int team_base = team * TEAM;
  const int64_t t = (tb * (kThreads / 64) + wave) * TPW + team;

  Task task = {0, 0, 0, -1};
  const bool has_task = t < ntasks;
  if (has_task) task = tasks[t];
  const int len = task.k1 - task.k0;

  // longest task in this wavefront (uniform loop bound, so the shuffles below stay convergent)
  int maxlen = len;
#pragma unroll
  for (int d = TEAM; d < 64; d <<= 1) maxlen = max(maxlen, __shfl_xor(maxlen, d));
  maxlen = __builtin_amdgcn_readfirstlane(maxlen);

  const int f0 = chunk * (LPR * VW) + fl * VW;
  const int nf = min(VW, max(0, F - f0));
  const float* __restrict__ xcol = X + f0;

  float acc[VW];
#pragma unroll
  for (int i = 0; i < VW; ++i) acc[i] = 0.f;

  int c = 0;
  float v = 0.f;
  if (tl < len) {
    c = __builtin_nontemporal_load(colidx + task.k0 + tl);
    v = __builtin_nontemporal_load(val + task.k0 + tl);
  }
  for (int base = 0; base < maxlen; base += TEAM) {
    int c_next = 0;
    float v_next = 0.f;
    if (base + TEAM + tl < len) {
      c_next = __builtin_nontemporal_load(colidx + task.k0 + base + TEAM + tl);
      v_next = __builtin_nontemporal_load(val + task.k0 + base + TEAM + tl);
    }
    const int remaining = maxlen - base;  // uniform
#pragma unroll
    for (int j0 = 0; j0 < LPR; j0 += U) {
      if (j0 * GPT >= remaining) break;
      float xs[U][VW];
      float vs[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int e = (j0 + u) * GPT + g;  // entry of this TEAM-chunk handled by my group
        const int cj = __shfl(c, team_base + e);
        vs[u] = __shfl(v, team_base + e);
        if (base + e < len && nf > 0) {
          load_row<VW>(xcol + (int64_t)cj * ldx, nf, xs[u]);
        } else {
#pragma unroll
          for (int i = 0; i < VW; ++i) xs[u][i] = 0.f;
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int i = 0; i < VW; ++i) acc[i] = fmaf(vs[u], xs[u][i], acc[i]);
    }
    c = c_next;
    v = v_next;
  }

  // fold the GPT lane groups of the team
#pragma unroll
  for (int d = LPR; d < TEAM; d <<= 1)
#pragma unroll
    for (int i = 0; i < VW; ++i) acc[i] += __shfl_xor(acc[i], d);

  if (has_task && g == 0 && nf > 0) {
    if (task.slot >= 0)
      store_out<VW>(partial + (int64_t)task.slot * ldp + f0, nf, acc, 0.f, MGGCN_EPI_NONE, false);
    else
      store_out<VW>(Y + (int64_t)task.row * ldy + f0, nf, acc, beta, epi, true);
  }
}

// Rows that were cut: add their partial sums in segment order.
__global__ __launch_bounds__(kThreads) void spmm_fixup(const FixRow* __restrict__ fix, int64_t nfix,
                                                        const float* __restrict__ partial,
                                                        int64_t ldp, int F, float beta, int epi,
                                                        float* __restrict__ Y, int64_t ldy) {
  const int64_t r = blockIdx.x;
  if (r >= nfix) return;
  const FixRow fr = fix[r];
  for (int f = threadIdx.x; f < F; f += kThreads) {
    float s = 0.f;
    for (int k = 0; k < fr.nslots; ++k) s += partial[(int64_t)(fr.slot0 + k) * ldp + f];
    float* dst = Y + (int64_t)fr.row * ldy + f;
    const float old = (beta != 0.f || epi == MGGCN_EPI_RELU_MASK) ? *dst : 0.f;
    *dst = apply_epilogue(s, old, beta, epi);
  }
}

struct LaunchArgs {
  const Task* tasks;
  int64_t ntasks;
  const int32_t* colidx;
  const float* val;
  const float* X;
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

template <int VW, int LPR, int GPT>
int launch_one(const LaunchArgs& a) {
  constexpr int TPW = 64 / (LPR * GPT);
  const int64_t teams_per_block = (kThreads / 64) * TPW;
  const int64_t blocks = ceil_div(a.ntasks, teams_per_block) * a.n_chunks;
  MGGCN_REQUIRE(blocks < ((int64_t)1 << 31), MGGCN_E_OVERFLOW, "SpMM grid of %lld blocks too large",
                (long long)blocks);
  spmm_tasks<VW, LPR, GPT><<<(unsigned)blocks, kThreads, 0, a.stream>>>(
      a.tasks, a.ntasks, a.colidx, a.val, a.X, a.ldx, a.F, a.n_chunks, a.beta, a.epi, a.Y, a.ldy,
      a.partial, a.ldp);
  MGGCN_LAUNCH_CHECK();
  return MGGCN_OK;
}

template <int VW, int LPR>
int launch_gpt(int gpt, const LaunchArgs& a) {
  switch (gpt) {
    case 1: return launch_one<VW, LPR, 1>(a);
    case 2: if constexpr (LPR * 2 <= 64) return launch_one<VW, LPR, 2>(a); break;
    case 4: if constexpr (LPR * 4 <= 64) return launch_one<VW, LPR, 4>(a); break;
    case 8: if constexpr (LPR * 8 <= 64) return launch_one<VW, LPR, 8>(a); break;
    case 16: if constexpr (LPR * 16 <= 64) return launch_one<VW, LPR, 16>(a); break;
    case 32: if constexpr (LPR * 32 <= 64) return launch_one<VW, LPR, 32>(a); break;
    case 64: if constexpr (LPR * 64 <= 64) return launch_one<VW, LPR, 64>(a); break;
    default: break;
  }
  return fail(MGGCN_E_UNSUPPORTED, "no SpMM kernel for %d lanes per row x %d groups", LPR, gpt);
}

template <int VW>
int launch_lpr(int lpr, int gpt, const LaunchArgs& a) {
  switch (lpr) {
    case 1: return launch_gpt<VW, 1>(gpt, a);
    case 2: return launch_gpt<VW, 2>(gpt, a);
    case 4: return launch_gpt<VW, 4>(gpt, a);
    case 8: return launch_gpt<VW, 8>(gpt, a);
    case 16: return launch_gpt<VW, 16>(gpt, a);
    case 32: return launch_gpt<VW, 32>(gpt, a);
    case 64: return launch_gpt<VW, 64>(gpt, a);
    default: break;
  }
  return fail(MGGCN_E_UNSUPPORTED, "no SpMM kernel for %d lanes per row", lpr);
}

int launch_any(int vw, int lpr, int gpt, const LaunchArgs& a) {
  switch (vw) {
    case 4: return launch_lpr<4>(lpr, gpt, a);
    case 2: return launch_lpr<2>(lpr, gpt, a);
    case 1: return launch_lpr<1>(lpr, gpt, a);
    default: break;
  }
  return fail(MGGCN_E_UNSUPPORTED, "no SpMM kernel for vector width %d", vw);
}

int pow2_ceil(int x) {
  int p = 1;
  while (p < x) p <<= 1;
  return p;
}

size_t carve_graph(const mggcn_graph* g, int32_t F_max, void* ws, Task** t0, FixRow** f0, Task** t1,
                   FixRow** f1, float** partial, int64_t* ldp_out) {
  Carver c(ws);
  Task* a = c.take<Task>(g->fwd.tasks.size() + 1);
  FixRow* b = c.take<FixRow>(g->fwd.fix.size() + 1);
  Task* a2 = nullptr;
  FixRow* b2 = nullptr;
  if (!g->symmetric) {
    a2 = c.take<Task>(g->bwd.tasks.size() + 1);
    b2 = c.take<FixRow>(g->bwd.fix.size() + 1);
  }
  const int64_t ldp = (int64_t)align_up((size_t)std::max(F_max, 1), 64);
  const int64_t slots = std::max(g->fwd.n_slots, g->symmetric ? 0 : g->bwd.n_slots);
  float* p = c.take<float>((size_t)(slots * ldp) + 64);
  if (t0) { *t0 = a; *f0 = b; *t1 = a2; *f1 = b2; *partial = p; *ldp_out = ldp; }
  return c.off;
}

}  // namespace
}  // namespace mggcn

using namespace mggcn;

extern "C" {

int mggcn_graph_create(int32_t n_rows, int32_t n_cols, const int32_t* rowptr, const int32_t* colidx,
                       const float* val, const int32_t* rowptr_t, const int32_t* colidx_t,
                       const float* val_t, int32_t seg_len, void* stream, mggcn_graph** out) {
  MGGCN_REQUIRE(out != nullptr, MGGCN_E_INVALID_ARG, "out is NULL");
  *out = nullptr;
  MGGCN_REQUIRE(n_rows >= 0 && n_cols >= 0, MGGCN_E_INVALID_ARG, "negative matrix size %d x %d",
                n_rows, n_cols);
  MGGCN_REQUIRE(rowptr != nullptr, MGGCN_E_INVALID_ARG, "rowptr is NULL");
  MGGCN_REQUIRE(seg_len >= 0 && seg_len <= (1 << 20), MGGCN_E_INVALID_ARG,
                "seg_len %d outside [0, 2^20]", seg_len);
  MGGCN_REQUIRE(rowptr_t != nullptr || n_rows == n_cols, MGGCN_E_INVALID_ARG,
                "a %d x %d matrix cannot be declared symmetric: pass its transpose", n_rows, n_cols);
  if (seg_len == 0) {
    seg_len = kDefaultSegLen;
    if (const char* e = std::getenv("MGGCN_SEG_LEN")) {
      const int v = std::atoi(e);
      if (v >= 8 && v <= (1 << 20)) seg_len = v;
    }
  }
  seg_len = std::max(seg_len, 8);
  hipStream_t s = as_stream(stream);

  mggcn_graph* g = new (std::nothrow) mggcn_graph;
  MGGCN_REQUIRE(g != nullptr, MGGCN_E_INVALID_ARG, "out of host memory");
  g->symmetric = (rowptr_t == nullptr);
  g->seg_len = seg_len;
  if (const char* e = std::getenv("MGGCN_CHUNK_LANES")) {
    const int v = std::atoi(e);
    if (v == 1 || v == 2 || v == 4 || v == 8 || v == 16 || v == 32 || v == 64) g->chunk_lanes = v;
  }

  auto setup = [&](Orientation* o, int32_t nr, int32_t nc, const int32_t* rp, const int32_t* ci,
                   const float* va) -> int {
    o->n_rows = nr; o->n_cols = nc; o->rowptr = rp; o->colidx = ci; o->val = va;
    std::vector<int32_t> h((size_t)nr + 1);
    MGGCN_HIP(hipMemcpyAsync(h.data(), rp, sizeof(int32_t) * ((size_t)nr + 1), hipMemcpyDeviceToHost, s));
    MGGCN_HIP(hipStreamSynchronize(s));
    MGGCN_REQUIRE(h[0] == 0, MGGCN_E_BAD_CSR, "rowptr[0] = %d, expected 0", h[0]);
    for (int32_t i = 0; i < nr; ++i)
      MGGCN_REQUIRE(h[(size_t)i + 1] >= h[i], MGGCN_E_BAD_CSR, "rowptr decreases at row %d", i);
    o->nnz = h[nr];
    MGGCN_REQUIRE(o->nnz == 0 || (ci && va), MGGCN_E_INVALID_ARG, "colidx / val is NULL");
    analyse(o, h, seg_len);
    return MGGCN_OK;
  };
  int rc = setup(&g->fwd, n_rows, n_cols, rowptr, colidx, val);
  if (!rc && !g->symmetric) rc = setup(&g->bwd, n_cols, n_rows, rowptr_t, colidx_t, val_t);
  if (!rc && !g->symmetric)
    if (g->bwd.nnz != g->fwd.nnz)
      rc = fail(MGGCN_E_BAD_CSR, "transpose has %lld entries, matrix has %lld",
                (long long)g->bwd.nnz, (long long)g->fwd.nnz);
  if (rc) { delete g; return rc; }
  *out = g;
  return MGGCN_OK;
}

size_t mggcn_graph_workspace_bytes(const mggcn_graph* g, int32_t F_max) {
  if (!g || F_max < 0) return 0;
  return carve_graph(g, F_max, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
}

int mggcn_graph_bind(mggcn_graph* g, int32_t F_max, void* ws, size_t ws_bytes, void* stream) {
  MGGCN_REQUIRE(g != nullptr, MGGCN_E_INVALID_ARG, "graph is NULL");
  MGGCN_REQUIRE(F_max >= 1, MGGCN_E_INVALID_ARG, "F_max = %d must be positive", F_max);
  MGGCN_REQUIRE(ws && aligned(ws, kWsAlign), MGGCN_E_WORKSPACE, "workspace is NULL or not 256-byte aligned");
  const size_t need = mggcn_graph_workspace_bytes(g, F_max);
  MGGCN_REQUIRE(ws_bytes >= need, MGGCN_E_WORKSPACE, "workspace too small: %zu bytes given, %zu needed",
                ws_bytes, need);
  hipStream_t s = as_stream(stream);
  Task *t0, *t1;
  FixRow *f0, *f1;
  carve_graph(g, F_max, ws, &t0, &f0, &t1, &f1, &g->d_partial, &g->ldp);
  auto upload = [&](Orientation* o, Task* dt, FixRow* df) -> int {
    o->d_tasks = dt;
    o->d_fix = df;
    if (!o->tasks.empty())
      MGGCN_HIP(hipMemcpyAsync(dt, o->tasks.data(), sizeof(Task) * o->tasks.size(), hipMemcpyHostToDevice, s));
    if (!o->fix.empty())
      MGGCN_HIP(hipMemcpyAsync(df, o->fix.data(), sizeof(FixRow) * o->fix.size(), hipMemcpyHostToDevice, s));
    return MGGCN_OK;
  };
  int rc = upload(&g->fwd, t0, f0);
  if (!rc && !g->symmetric) rc = upload(&g->bwd, t1, f1);
  if (rc) return rc;
  MGGCN_HIP(hipStreamSynchronize(s));  // host vectors may be touched again after return
  g->F_bound = F_max;
  g->bound = true;
  return MGGCN_OK;
}

int mggcn_graph_destroy(mggcn_graph* g) {
  delete g;
  return MGGCN_OK;
}

int mggcn_spmm(const mggcn_graph* g, int op, const float* X, int64_t ldx, int32_t F, float beta,
               int epilogue, float* Y, int64_t ldy, void* stream) {
  MGGCN_REQUIRE(g != nullptr, MGGCN_E_INVALID_ARG, "graph is NULL");
  MGGCN_REQUIRE(op == MGGCN_OP_N || op == MGGCN_OP_T, MGGCN_E_INVALID_ARG, "unknown op %d", op);
  MGGCN_REQUIRE(F >= 0, MGGCN_E_INVALID_ARG, "F = %d is negative", F);
  MGGCN_REQUIRE(ldx >= F && ldy >= F, MGGCN_E_INVALID_ARG, "leading dimension (ldx %lld, ldy %lld) < F %d",
                (long long)ldx, (long long)ldy, F);
  MGGCN_REQUIRE(beta == 0.f || beta == 1.f, MGGCN_E_INVALID_ARG, "beta must be 0 or 1");
  MGGCN_REQUIRE(epilogue == MGGCN_EPI_NONE || epilogue == MGGCN_EPI_RELU || epilogue == MGGCN_EPI_RELU_MASK,
                MGGCN_E_INVALID_ARG, "unknown epilogue %d", epilogue);
  MGGCN_REQUIRE(!(epilogue == MGGCN_EPI_RELU_MASK && beta != 0.f), MGGCN_E_INVALID_ARG,
                "RELU_MASK cannot be combined with beta = 1");
  MGGCN_REQUIRE(g->bound, MGGCN_E_WORKSPACE, "graph is not bound to a workspace");
  MGGCN_REQUIRE(F <= g->F_bound, MGGCN_E_WORKSPACE, "F = %d exceeds the bound width %d", F, g->F_bound);
  const Orientation& o = (op == MGGCN_OP_N || g->symmetric) ? g->fwd : g->bwd;
  if (F == 0 || o.n_rows == 0) return MGGCN_OK;
  MGGCN_REQUIRE(X != nullptr || o.nnz == 0, MGGCN_E_INVALID_ARG, "X is NULL");
  MGGCN_REQUIRE(Y != nullptr, MGGCN_E_INVALID_ARG, "Y is NULL");

  int vw = 1;
  if (aligned(X, 16) && aligned(Y, 16) && ldx % 4 == 0 && ldy % 4 == 0) vw = 4;
  else if (aligned(X, 8) && aligned(Y, 8) && ldx % 2 == 0 && ldy % 2 == 0) vw = 2;
  int lpr = std::min(64, pow2_ceil((int)ceil_div(F, vw)));
  if (g->chunk_lanes > 0) lpr = std::min(lpr, g->chunk_lanes);
  const int n_chunks = (int)ceil_div(F, lpr * vw);
  const int gpt_max = 64 / lpr;

  LaunchArgs a;
  a.colidx = o.colidx; a.val = o.val; a.X = X; a.ldx = ldx; a.F = F; a.n_chunks = n_chunks;
  a.beta = beta; a.epi = epilogue; a.Y = Y; a.ldy = ldy; a.partial = g->d_partial; a.ldp = g->ldp;
  a.stream = as_stream(stream);

  // bins of tasks by length; tasks are sorted longest first, so every bin is a contiguous range
  const int64_t ntasks = (int64_t)o.tasks.size();
  int top = 0;
  while ((1 << (top + 1)) <= gpt_max) ++top;  // gpt_max = 1 << top
  int64_t begin = 0;
  for (int i = top; i >= 0; --i) {
    const int64_t end = (i == 0) ? ntasks : o.cnt_ge[i];  // length >= 8 << i  => gpt = 1 << i
    if (end > begin) {
      a.tasks = o.d_tasks + begin;
      a.ntasks = end - begin;
      const int rc = launch_any(vw, lpr, 1 << i, a);
      if (rc) return rc;
      begin = end;
    }
  }
  if (!o.fix.empty()) {
    spmm_fixup<<<(unsigned)o.fix.size(), kThreads, 0, a.stream>>>(o.d_fix, (int64_t)o.fix.size(),
                                                                  g->d_partial, g->ldp, F, beta,
                                                                  epilogue, Y, ldy);
    MGGCN_LAUNCH_CHECK();
  }
  return MGGCN_OK;
}

}  // extern "C"
