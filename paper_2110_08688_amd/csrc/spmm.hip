// CSR SpMM  Y = epilogue( op(A^) X + beta Y )  for gfx950 -- the product that takes most of a
// GCN epoch (Eq. 6 forward, Eq. 9 backward of the paper).
//
// Work decomposition (done once per graph, the graph being fixed for all epochs; built on the device
// when the handle is bound to its workspace, tasks.hip):
//   every row is cut into segments of at most seg_len entries; a segment is a task.  Tasks are
//   ordered longest first.  A row with one segment is written straight to Y; the segments of a
//   cut row go to a partial-sum table and a second small kernel adds them in segment order, so
//   the result never depends on timing (no floating-point atomics).
//
// Column panels (the "blocking effect" the paper observes for column tiles, and the same algebra
// as its stage loop C += A^{ij} H^j): on a dense-ish graph the gathered operand X is far larger
// than the 8 x 4 MB of L2, and throughput follows how much of it the caches hold.  The column
// range is therefore cut into P equal panels; columns being sorted inside a row, the entries of
// a (row, panel) pair are a contiguous sub-range, so no data moves.  Panels run as successive
// launches on the stream, each adding into Y (beta = 1 after a row's first panel, epilogue at its
// last): all wavefronts in flight then gather from the same 1/P of X.  The price is one
// read-modify-write of Y per panel, so P is capped by the average row length.  Tables are kept
// for P = 2, 4, 8, ... and each product picks the count that brings one panel of its operand to
// about 16 MiB; an operand too wide even for the largest count is also walked in feature slices.
//
// Kernel mapping (wave64), see spmm_kernel.h:
//   the feature dimension runs along lanes: LPR lanes x VW elements cover one feature chunk of a
//   dense row, so a gathered row is read with 16-byte loads that are contiguous across lanes.
//   A team of LPR*GPT lanes owns one task: GPT lane groups walk the segment's entries
//   interleaved, and their accumulators are folded with xor-shuffles at the end.  Column
//   indices and values are fetched TEAM entries at a time with one coalesced streaming load
//   and handed to the groups by ds_bpermute.  Long tasks get the whole wave (GPT = 64/LPR);
//   short ones get narrower teams so that several rows share a wave; all length bins of a pass
//   run in one launch.  A row wider than one wave's reach (more than 64 lanes x VW elements)
//   is covered by several feature chunks, interleaved over blockIdx.
#include "spmm_kernel.h"

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

namespace mggcn {
namespace {

constexpr int kThreads = kSpmmThreads;
constexpr int kDefaultSegLen = 2048;

// Entry offset at which each row crosses each panel boundary: cuts[i * n_cuts + c] = first entry
// of row i whose column is >= (c + 1) * width (columns are ascending inside a row).  One thread per
// (row, boundary), a binary search each.
template <typename IT>
__global__ __launch_bounds__(kSpmmThreads) void panel_cuts(int32_t n_rows, int32_t n_cols, const IT* __restrict__ rowptr,
                                                            const int32_t* __restrict__ colidx, int64_t width,
                                                            int32_t n_cuts, uint32_t* __restrict__ cuts) {
  const int64_t idx = (int64_t)blockIdx.x * kSpmmThreads + threadIdx.x;
  if (idx >= (int64_t)n_rows * n_cuts) return;
  const int64_t i = idx / n_cuts;
  const int32_t c = (int32_t)(idx % n_cuts);
  const int64_t bound = min((int64_t)(c + 1) * width, (int64_t)n_cols);
  int64_t lo = rowptr[i], hi = rowptr[i + 1];
  while (lo < hi) {
    const int64_t mid = (lo + hi) >> 1;
    if (colidx[mid] < bound) lo = mid + 1; else hi = mid;
  }
  cuts[idx] = (uint32_t)lo;
}

// A column index outside [0, n_cols) would send a gather outside X: found here, once, instead.
__global__ __launch_bounds__(kSpmmThreads) void check_columns(int64_t nnz, int32_t n_cols,
                                                               const int32_t* __restrict__ colidx,
                                                               uint32_t* __restrict__ bad) {
  const int64_t k = (int64_t)blockIdx.x * kSpmmThreads + threadIdx.x;
  if (k < nnz && (uint32_t)colidx[k] >= (uint32_t)n_cols) *bad = 1u;  // every writer stores the same value
}

// Row offsets checked and table sizes bounded in one pass over the rows, on the device: every workgroup
// writes its own sums to host-visible memory (no atomics), the host adds the few hundred of them up.
constexpr int kMaxForms = 8;       // the single-pass table + up to seven panel tables
constexpr int kRowCheckBlocks = 512;
struct FormList { int32_t n; int32_t panels[kMaxForms]; };
struct RowCheckOut {               // one per workgroup
  int64_t first_decreasing, first_too_long;  // row index, or -1
  int64_t tasks[kMaxForms], fix[kMaxForms], slots[kMaxForms];
};

// Upper bounds of a table's size from the row lengths alone: a row of L entries in P panels has at most
// min(P, L) non-empty ranges (one empty range if L = 0); a range of r entries makes ceil(r / seg_len)
// <= r / seg_len + 1 tasks, and is cut (one fix-up record, its tasks writing to slots) only if r > seg_len.
__host__ __device__ inline void row_bounds(int64_t len, int64_t P, int32_t seg_len, int64_t* tasks, int64_t* fix, int64_t* slots) {
  *tasks += len == 0 ? 1 : (P < len ? P : len) + len / seg_len;
  if (len > seg_len) {
    const int64_t most = len / ((int64_t)seg_len + 1), cut = P < most ? P : most;
    *fix += cut;
    *slots += len / seg_len + cut;
  }
}

template <typename IT>
__global__ __launch_bounds__(kSpmmThreads) void check_rows(int64_t n_rows, const IT* __restrict__ rowptr, int32_t seg_len,
                                                            FormList forms, RowCheckOut* __restrict__ out) {
  int64_t dec = -1, big = -1, acc[3 * kMaxForms];
#pragma unroll
  for (int k = 0; k < 3 * kMaxForms; ++k) acc[k] = 0;
  for (int64_t i = (int64_t)blockIdx.x * kSpmmThreads + threadIdx.x; i < n_rows; i += (int64_t)gridDim.x * kSpmmThreads) {
    const int64_t len = (int64_t)rowptr[i + 1] - (int64_t)rowptr[i];
    if (len < 0) { if (dec < 0) dec = i; continue; }
    if (len > (int64_t)kTaskLenMask && big < 0) big = i;
#pragma unroll
    for (int f = 0; f < kMaxForms; ++f)
      if (f < forms.n) row_bounds(len, forms.panels[f], seg_len, &acc[f], &acc[kMaxForms + f], &acc[2 * kMaxForms + f]);
  }
  // block reduction: sums of the bounds, smallest offending row (as unsigned, -1 is the largest)
  __shared__ int64_t red[kSpmmThreads / 64][3 * kMaxForms + 2];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint64_t udec = (uint64_t)dec, ubig = (uint64_t)big;
  for (int d = 1; d < 64; d <<= 1) {
    const uint64_t a = __shfl_xor((unsigned long long)udec, d), b = __shfl_xor((unsigned long long)ubig, d);
    udec = a < udec ? a : udec;
    ubig = b < ubig ? b : ubig;
#pragma unroll
    for (int k = 0; k < 3 * kMaxForms; ++k) acc[k] += (int64_t)__shfl_xor((long long)acc[k], d);
  }
  if (lane == 0) {
    for (int k = 0; k < 3 * kMaxForms; ++k) red[wave][k] = acc[k];
    red[wave][3 * kMaxForms] = (int64_t)udec;
    red[wave][3 * kMaxForms + 1] = (int64_t)ubig;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    RowCheckOut o;
    uint64_t d0 = ~0ull, b0 = ~0ull;
    for (int k = 0; k < 3 * kMaxForms; ++k) acc[k] = 0;
    for (int w = 0; w < kSpmmThreads / 64; ++w) {
      for (int k = 0; k < 3 * kMaxForms; ++k) acc[k] += red[w][k];
      d0 = (uint64_t)red[w][3 * kMaxForms] < d0 ? (uint64_t)red[w][3 * kMaxForms] : d0;
      b0 = (uint64_t)red[w][3 * kMaxForms + 1] < b0 ? (uint64_t)red[w][3 * kMaxForms + 1] : b0;
    }
    o.first_decreasing = (int64_t)d0;
    o.first_too_long = (int64_t)b0;
    for (int f = 0; f < kMaxForms; ++f) { o.tasks[f] = acc[f]; o.fix[f] = acc[kMaxForms + f]; o.slots[f] = acc[2 * kMaxForms + f]; }
    out[blockIdx.x] = o;
  }
}

int pow2_floor(int64_t x) {
  int p = 1;
  while ((int64_t)p * 2 <= x) p <<= 1;
  return p;
}

// Most column panels a matrix affords: every panel costs one more read-modify-write of the output,
// which an average row of ~50 entries does not earn back even with 2 panels, while ~490 entries
// carry 16 (measured).
int32_t max_panels(int32_t n_rows, int64_t nnz) {
  if (n_rows <= 0 || nnz <= 0) return 1;
  return (int32_t)std::min<int64_t>(pow2_floor(std::max<int64_t>(1, nnz / n_rows / 30)), 32);
}

int pow2_ceil(int x) {
  int p = 1;
  while (p < x) p <<= 1;
  return p;
}

// Panel form for a product whose gathered operand has n_cols rows of F elements of elem_bytes:
// the smallest power-of-two panel count that brings one panel of the operand down to
// the target size (a panel that all wavefronts in flight share then lives in L2 / Infinity
// Cache), among the forms built.
// Target size of one panel of the gathered operand.  Measured best on MI355X: about 16 MiB for
// 2-byte elements and 12 MiB for 4-byte ones -- the read-modify-write of the fp32 output that every
// panel costs weighs twice as much against a gather of half the bytes.
int64_t panel_target(const mggcn_graph* g, int elem_bytes) {
  return std::max<int64_t>(elem_bytes >= 4 ? g->panel_bytes / 4 * 3 : g->panel_bytes, 1);
}

const TaskSet* pick_panels(const mggcn_graph* g, const Orientation& o, int32_t F, int elem_bytes, int epilogue) {
  // the in-place ReLU' mask needs the old Y at every write, which only the single-panel form provides
  if (o.panelled.empty() || epilogue == MGGCN_EPI_RELU_MASK) return &o.flat;
  if (g->panels_fixed) return &o.panelled.front();
  const int64_t bytes = (int64_t)o.n_cols * F * elem_bytes;
  const int want = pow2_ceil((int)std::min<int64_t>(ceil_div(bytes, panel_target(g, elem_bytes)), 1 << 20));
  if (want <= 1) return &o.flat;
  const TaskSet* best = &o.panelled.front();
  for (const TaskSet& ts : o.panelled)
    if (ts.n_panels <= want) best = &ts;  // ascending panel counts: the largest not above `want`
  return best;
}

// ---------------------------------------------------------------------------------------
// device code
// ---------------------------------------------------------------------------------------

// Rows that were cut: add their partial sums in segment order.
__global__ __launch_bounds__(kThreads) void spmm_fixup(const FixRow* __restrict__ fix, int64_t nfix,
                                                        const float* __restrict__ partial,
                                                        int64_t ldp, int F, float beta, int epi,
                                                        float* __restrict__ Y, int64_t ldy) {
  const int64_t r = blockIdx.x;
  if (r >= nfix) return;
  const FixRow fr = fix[r];
  if (!(fr.flags & kTaskFirst)) beta = 1.f;
  if (!(fr.flags & kTaskLast)) epi = MGGCN_EPI_NONE;
  for (int f = threadIdx.x; f < F; f += kThreads) {
    float s = 0.f;
    for (int k = 0; k < fr.nslots; ++k) s += partial[(int64_t)(fr.slot0 + k) * ldp + f];
    float* dst = Y + (int64_t)fr.row * ldy + f;
    const float old = (beta != 0.f || epi == MGGCN_EPI_RELU_MASK) ? *dst : 0.f;
    *dst = apply_epilogue(s, old, beta, epi);
  }
}

// Rows of op(A^) without a single entry, beta = 0: their result is zero whatever the epilogue, and
// their tasks are the tail of a pass's task list (zero length sorts last; rows ascending).  They
// are written here at the rate of a fill instead of each taking a lane team of the gather kernel
// through its whole prologue: 79 M such rows of 128 floats took 10.9 ms there, a plain fill of the
// same memory 6.2 ms (the transposed product of a 13.9 M x 111 M row block has that many).
// One lane per VW floats of a row, `lanes` (a power of two, at most 64) per row; a wavefront takes up to
// 64 consecutive tasks, reads each task once (one lane each) and hands the row numbers round by shuffles.
template <int VW>
__global__ __launch_bounds__(kThreads) void spmm_zero_rows(const Task* __restrict__ tasks, int64_t n, int F, int lanes_log2,
                                                            int rows_per_team, float* __restrict__ Y, int64_t ldy,
                                                            float* __restrict__ partial, int64_t ldp) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int tpw = 64 >> lanes_log2;  // teams (rows side by side) per wavefront
  const int team = lane >> lanes_log2, fl = lane & ((1 << lanes_log2) - 1);
  const int per_wave = tpw * rows_per_team;  // <= 64
  const int64_t base = ((int64_t)blockIdx.x * (kThreads / 64) + wave) * per_wave;
  int32_t my_row = 0, my_slot = -1;
  if (lane < per_wave && base + lane < n) {
    my_row = tasks[base + lane].row;
    my_slot = tasks[base + lane].slot;
  }
  const int f0 = fl * VW;
  const int nf = min(VW, F - f0);
  const float zero[VW] = {};
  for (int j = 0; j < rows_per_team; ++j) {
    const int r = j * tpw + team;  // the same for all lanes of a team; every lane takes part in the shuffles
    const int32_t row = __shfl(my_row, r), slot = __shfl(my_slot, r);
    if (base + r < n && nf > 0) {
      // a zero-length piece of a cut row (its sum lives in the partial table) is zero there
      float* dst = slot < 0 ? Y + (int64_t)row * ldy + f0 : partial + (int64_t)slot * ldp + f0;
      store_out<VW>(dst, nf, zero, 0.f, MGGCN_EPI_NONE, false, slot < 0);
    }
  }
}

// false: the shape does not fit the fill kernel (the rows stay with the gather launch)
bool zero_rows_shape(const float* Y, int64_t ldy, int F, int* vw, int* lanes_log2, int* rows_per_team) {
  *vw = 1;
  if (aligned(Y, 16) && ldy % 4 == 0) *vw = 4;
  else if (aligned(Y, 8) && ldy % 2 == 0) *vw = 2;
  *lanes_log2 = 0;
  while ((1 << *lanes_log2) * *vw < F && *lanes_log2 < 6) ++*lanes_log2;
  if ((int64_t)(1 << *lanes_log2) * *vw < F) return false;
  *rows_per_team = std::min(8, 64 / (64 >> *lanes_log2));
  return true;
}

int launch_zero_rows(const Task* tasks, int64_t n, int F, float* Y, int64_t ldy, float* partial, int64_t ldp, hipStream_t s) {
  int vw, lanes_log2, rows_per_team;
  MGGCN_REQUIRE(zero_rows_shape(Y, ldy, F, &vw, &lanes_log2, &rows_per_team), MGGCN_E_OVERFLOW,
                "F = %d too wide for the zero-row kernel", F);
  const int64_t rows_per_block = (int64_t)(kThreads / 64) * (64 >> lanes_log2) * rows_per_team;
  const int64_t blocks = ceil_div(n, rows_per_block);
  MGGCN_REQUIRE(blocks < ((int64_t)1 << 31), MGGCN_E_OVERFLOW, "zero-row grid too large");
#define MGGCN_ZERO_ROWS(VW) \
  spmm_zero_rows<VW><<<(unsigned)blocks, kThreads, 0, s>>>(tasks, n, F, lanes_log2, rows_per_team, Y, ldy, partial, ldp)
  if (vw == 4) MGGCN_ZERO_ROWS(4);
  else if (vw == 2) MGGCN_ZERO_ROWS(2);
  else MGGCN_ZERO_ROWS(1);
#undef MGGCN_ZERO_ROWS
  MGGCN_LAUNCH_CHECK();
  return MGGCN_OK;
}

int launch_any_f32(int vw, int lpr, const LaunchArgs& a) {
  switch (vw) {
    case 4: return launch_lpr<float, 4>(lpr, a);
    case 2: return launch_lpr<float, 2>(lpr, a);
    case 1: return launch_lpr<float, 1>(lpr, a);
    default: break;
  }
  return fail(MGGCN_E_UNSUPPORTED, "no SpMM kernel for vector width %d", vw);
}

struct GraphCarve {
  std::vector<Task*> tasks[2];   // per orientation: flat form first, then the panel forms
  std::vector<FixRow*> fix[2];
  float* partial;
  int64_t ldp;
  uint32_t* cuts;                // build scratch: panel boundaries of every row of one orientation
  void* build;                   // build scratch of one table at a time
};

size_t carve_graph(const mggcn_graph* g, int32_t F_max, void* ws, GraphCarve* out) {
  Carver c(ws);
  GraphCarve gc = {};
  int64_t slots = 0;
  size_t cut_words = 1, build_bytes = kWsAlign;
  const Orientation* os[2] = {&g->fwd, g->symmetric ? nullptr : &g->bwd};
  for (int o = 0; o < 2; ++o) {
    if (!os[o]) continue;
    std::vector<const TaskSet*> sets = {&os[o]->flat};
    for (const TaskSet& ts : os[o]->panelled) sets.push_back(&ts);
    for (const TaskSet* ts : sets) {
      gc.tasks[o].push_back(c.take<Task>((size_t)ts->max_tasks + 1));
      gc.fix[o].push_back(c.take<FixRow>((size_t)ts->max_fix + 1));
      slots = std::max(slots, ts->max_slots);
      build_bytes = std::max(build_bytes, task_build_scratch_bytes(os[o]->n_rows, ts->n_panels, ts->max_tasks));
    }
    if (os[o]->finest > 1) cut_words = std::max(cut_words, (size_t)os[o]->n_rows * (size_t)(os[o]->finest - 1));
  }
  gc.ldp = (int64_t)align_up((size_t)std::max(F_max, 1), 64);
  gc.partial = c.take<float>((size_t)(slots * gc.ldp) + 64);
  // scratch of mggcn_graph_bind, free for nothing else afterwards (the tables are built once per binding)
  gc.cuts = c.take<uint32_t>(cut_words);
  gc.build = c.take<char>(build_bytes);
  if (out) *out = std::move(gc);
  return c.off;
}

// All tables of one orientation, built on the device into the carved workspace.
template <typename IT>
int build_tables(const mggcn_graph* g, Orientation* o, const GraphCarve& gc, int which, hipStream_t s) {
  const IT* rp = static_cast<const IT*>(o->rowptr);
  const int32_t n_cuts = o->finest - 1;
  if (n_cuts > 0 && o->n_rows > 0) {
    // where every row crosses the boundaries of the finest panels; coarser tables use every 2nd, 4th, ... of them
    const int64_t width = ceil_div(std::max(o->n_cols, 1), o->finest);
    const int64_t items = (int64_t)o->n_rows * n_cuts;
    MGGCN_REQUIRE(ceil_div(items, kThreads) < ((int64_t)1 << 31), MGGCN_E_OVERFLOW, "panel boundary grid too large");
    panel_cuts<IT><<<(unsigned)ceil_div(items, kThreads), kThreads, 0, s>>>(o->n_rows, o->n_cols, rp, o->colidx, width, n_cuts,
                                                                           gc.cuts);
    MGGCN_LAUNCH_CHECK();
  }
  int rc = build_task_set_device<IT>(&o->flat, o->n_rows, rp, nullptr, 0, 0, g->seg_len, gc.tasks[which][0], gc.fix[which][0],
                                     gc.build, s);
  for (size_t k = 0; !rc && k < o->panelled.size(); ++k) {
    TaskSet& ts = o->panelled[k];
    rc = build_task_set_device<IT>(&ts, o->n_rows, rp, gc.cuts, n_cuts, o->finest / ts.n_panels, g->seg_len,
                                   gc.tasks[which][k + 1], gc.fix[which][k + 1], gc.build, s);
  }
  return rc;
}

}  // namespace
}  // namespace mggcn

namespace mggcn {
namespace {

template <typename IT>
int graph_create_impl(int32_t n_rows, int32_t n_cols, const IT* rowptr, const int32_t* colidx, const float* val,
                      const IT* rowptr_t, const int32_t* colidx_t, const float* val_t, int32_t seg_len,
                      int32_t n_panels, void* stream, mggcn_graph** out) {
  MGGCN_REQUIRE(out != nullptr, MGGCN_E_INVALID_ARG, "out is NULL");
  *out = nullptr;
  MGGCN_REQUIRE(n_rows >= 0 && n_cols >= 0, MGGCN_E_INVALID_ARG, "negative matrix size %d x %d",
                n_rows, n_cols);
  MGGCN_REQUIRE(rowptr != nullptr, MGGCN_E_INVALID_ARG, "rowptr is NULL");
  MGGCN_REQUIRE(seg_len >= 0 && seg_len <= (1 << 20), MGGCN_E_INVALID_ARG,
                "seg_len %d outside [0, 2^20]", seg_len);
  MGGCN_REQUIRE(rowptr_t != nullptr || n_rows == n_cols, MGGCN_E_INVALID_ARG,
                "a %d x %d matrix cannot be declared symmetric: pass its transpose", n_rows, n_cols);
  MGGCN_REQUIRE(n_panels >= 0 && n_panels <= 64, MGGCN_E_INVALID_ARG, "n_panels %d outside [0, 64]",
                n_panels);
  if (seg_len == 0) seg_len = kDefaultSegLen;
  seg_len = std::max(seg_len, 8);
  hipStream_t s = as_stream(stream);

  mggcn_graph* g = new (std::nothrow) mggcn_graph;
  MGGCN_REQUIRE(g != nullptr, MGGCN_E_NO_MEMORY, "out of host memory");
  g->symmetric = (rowptr_t == nullptr);
  g->seg_len = seg_len;
  g->panel_bytes = 16ll << 20;
  g->panels_fixed = n_panels > 1;
  auto setup = [&](Orientation* o, int32_t nr, int32_t nc, const IT* rp, const int32_t* ci,
                   const float* va) -> int {
    o->n_rows = nr; o->n_cols = nc; o->rowptr = rp; o->wide = sizeof(IT) == 8; o->colidx = ci; o->val = va;
    IT ends[2] = {0, 0};  // rowptr[0], rowptr[nr]
    MGGCN_HIP(hipMemcpyAsync(&ends[0], rp, sizeof(IT), hipMemcpyDeviceToHost, s));
    MGGCN_HIP(hipMemcpyAsync(&ends[1], rp + nr, sizeof(IT), hipMemcpyDeviceToHost, s));
    MGGCN_HIP(hipStreamSynchronize(s));
    MGGCN_REQUIRE(ends[0] == 0, MGGCN_E_BAD_CSR, "rowptr[0] = %lld, expected 0", (long long)ends[0]);
    MGGCN_REQUIRE(ends[1] >= 0, MGGCN_E_BAD_CSR, "rowptr[%d] = %lld is negative", nr, (long long)ends[1]);
    o->nnz = (int64_t)ends[1];
    MGGCN_REQUIRE(o->nnz < ((int64_t)1 << 32), MGGCN_E_OVERFLOW,
                  "%lld entries: entry offsets are held in 32 unsigned bits", (long long)o->nnz);
    MGGCN_REQUIRE(o->nnz == 0 || (ci && va), MGGCN_E_INVALID_ARG, "colidx / val is NULL");
    struct Pinned {  // freed on every way out, a failed allocation of the tables included
      uint32_t* p = nullptr;
      ~Pinned() { if (p) (void)hipHostFree(p); }
    };
    if (o->nnz > 0) {
      Pinned bad;
      MGGCN_HIP(hipHostMalloc(reinterpret_cast<void**>(&bad.p), sizeof(uint32_t), hipHostMallocDefault));
      *bad.p = 0u;
      check_columns<<<(unsigned)ceil_div(o->nnz, kThreads), kThreads, 0, s>>>(o->nnz, nc, ci, bad.p);
      hipError_t e = hipGetLastError();
      if (e == hipSuccess) e = hipStreamSynchronize(s);
      if (e != hipSuccess) return fail(MGGCN_E_HIP, "column index check failed: %s", hipGetErrorString(e));
      MGGCN_REQUIRE(*bad.p == 0u, MGGCN_E_BAD_CSR, "a column index lies outside [0, %d)", nc);
    }
    // The tables themselves are built on the device when the handle is bound; here only their forms
    // (one panel; n_panels panels, or 2, 4, 8, ... as far as the average row length affords, over one
    // common finest width) and the upper bounds of their sizes, which the workspace query needs.
    o->flat.n_panels = 1;
    const int32_t Pmax = n_panels > 0 ? n_panels : max_panels(nr, o->nnz);
    o->finest = 1;
    if (Pmax > 1 && nr > 0) {
      o->finest = Pmax;
      for (int32_t P = n_panels > 0 ? n_panels : 2; P <= Pmax; P *= 2) {
        o->panelled.emplace_back();
        o->panelled.back().n_panels = P;
      }
    }
    std::vector<TaskSet*> sets = {&o->flat};
    for (TaskSet& t : o->panelled) sets.push_back(&t);
    MGGCN_REQUIRE(sets.size() <= (size_t)kMaxForms, MGGCN_E_UNSUPPORTED, "%zu table forms", sets.size());
    if (nr > 0) {
      FormList forms = {};
      forms.n = (int32_t)sets.size();
      for (size_t f = 0; f < sets.size(); ++f) forms.panels[f] = sets[f]->n_panels;
      struct PinnedOut {
        RowCheckOut* p = nullptr;
        ~PinnedOut() { if (p) (void)hipHostFree(p); }
      } res;
      MGGCN_HIP(hipHostMalloc(reinterpret_cast<void**>(&res.p), sizeof(RowCheckOut) * kRowCheckBlocks, hipHostMallocDefault));
      const int blocks = (int)std::min<int64_t>(kRowCheckBlocks, ceil_div(nr, kThreads));
      check_rows<IT><<<blocks, kThreads, 0, s>>>(nr, rp, seg_len, forms, res.p);
      hipError_t e = hipGetLastError();
      if (e == hipSuccess) e = hipStreamSynchronize(s);
      if (e != hipSuccess) return fail(MGGCN_E_HIP, "row offset check failed: %s", hipGetErrorString(e));
      int64_t dec = -1, big = -1;
      for (int b = 0; b < blocks; ++b) {
        const RowCheckOut& r = res.p[b];
        if (r.first_decreasing >= 0 && (dec < 0 || r.first_decreasing < dec)) dec = r.first_decreasing;
        if (r.first_too_long >= 0 && (big < 0 || r.first_too_long < big)) big = r.first_too_long;
        for (size_t f = 0; f < sets.size(); ++f) {
          sets[f]->max_tasks += r.tasks[f];
          sets[f]->max_fix += r.fix[f];
          sets[f]->max_slots += r.slots[f];
        }
      }
      MGGCN_REQUIRE(dec < 0, MGGCN_E_BAD_CSR, "rowptr decreases at row %lld", (long long)dec);
      MGGCN_REQUIRE(big < 0, MGGCN_E_OVERFLOW, "row %lld holds more than 2^29 - 1 entries", (long long)big);
    }
    for (TaskSet* ts : sets)
      MGGCN_REQUIRE(ts->max_tasks < ((int64_t)1 << 32), MGGCN_E_OVERFLOW, "%lld row segments: positions are held in 32 unsigned bits",
                    (long long)ts->max_tasks);
    return MGGCN_OK;
  };
  int rc = guarded([&] { return setup(&g->fwd, n_rows, n_cols, rowptr, colidx, val); });
  if (!rc && !g->symmetric) rc = guarded([&] { return setup(&g->bwd, n_cols, n_rows, rowptr_t, colidx_t, val_t); });
  if (!rc && !g->symmetric)
    if (g->bwd.nnz != g->fwd.nnz)
      rc = fail(MGGCN_E_BAD_CSR, "transpose has %lld entries, matrix has %lld",
                (long long)g->bwd.nnz, (long long)g->fwd.nnz);
  if (rc) { delete g; return rc; }
  *out = g;
  return MGGCN_OK;
}

}  // namespace

int spmm_check_args(const mggcn_graph* g, int op, const void* X, int64_t ldx, int elem_bytes, int32_t F,
                    float beta, int epilogue, const float* Y, int64_t ldy) {
  MGGCN_REQUIRE(g != nullptr, MGGCN_E_INVALID_ARG, "graph is NULL");
  MGGCN_REQUIRE(op == MGGCN_OP_N || op == MGGCN_OP_T, MGGCN_E_INVALID_ARG, "unknown op %d", op);
  MGGCN_REQUIRE(F >= 0, MGGCN_E_INVALID_ARG, "F = %d is negative", F);
  MGGCN_REQUIRE(ldx >= F && ldy >= F, MGGCN_E_INVALID_ARG, "leading dimension (ldx %lld, ldy %lld) < F %d",
                (long long)ldx, (long long)ldy, F);
  MGGCN_REQUIRE(ldx < ((int64_t)1 << 30), MGGCN_E_OVERFLOW, "ldx %lld: a row of X must be shorter than 4 GiB",
                (long long)ldx);
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
  if (X != nullptr && o.n_cols > 0) {  // rows of Y are written while rows of X are still being gathered
    const char* xb = static_cast<const char*>(X);
    // the wide gather path reads whole 16-byte vectors: a row of X is read up to F rounded up to
    // 4 floats (8 bfloat16), which lies inside its leading dimension
    const size_t per_vec = 16 / (size_t)elem_bytes;
    const size_t x_cols = std::min<size_t>((size_t)ldx, align_up((size_t)F, per_vec));
    const char* xe = xb + ((size_t)(o.n_cols - 1) * (size_t)ldx + x_cols) * (size_t)elem_bytes;
    const char* yb = reinterpret_cast<const char*>(Y);
    const char* ye = yb + ((size_t)(o.n_rows - 1) * (size_t)ldy + (size_t)F) * sizeof(float);
    MGGCN_REQUIRE(xe <= yb || ye <= xb, MGGCN_E_INVALID_ARG, "X and Y overlap");
  }
  return MGGCN_OK;
}

namespace {

constexpr int64_t kZeroRowsWorthALaunch = 1 << 16;  // fewer rows without entries stay in the gather launch

// One product over the first F columns of X / Y with the given task tables.
int spmm_run_slice(const mggcn_graph* g, const Orientation& o, const TaskSet& ts, const void* X, int64_t ldx,
                   int vw, int32_t F, float beta, int epilogue, float* Y, int64_t ldy, void* stream,
                   SpmmLaunchFn launch) {
  int lpr = std::min(64, pow2_ceil((int)ceil_div(F, vw)));
  if (g->chunk_lanes > 0) lpr = std::min(lpr, g->chunk_lanes);
  const int n_chunks = (int)ceil_div(F, lpr * vw);
  const int gpt_max = 64 / lpr;

  LaunchArgs a;
  a.colidx = o.colidx; a.val = o.val; a.X = X; a.ldx = ldx; a.F = F; a.n_chunks = n_chunks;
  a.beta = beta; a.epi = epilogue; a.Y = Y; a.ldy = ldy; a.partial = g->d_partial; a.ldp = g->ldp;
  a.stream = as_stream(stream);

  int top = 0;
  while ((1 << (top + 1)) <= gpt_max) ++top;  // gpt_max = 1 << top
  for (int32_t p = 0; p < ts.n_panels; ++p) {
    // bins of tasks by length; tasks are sorted longest first, so every bin is a contiguous range
    int64_t ntasks = ts.task_begin[(size_t)p + 1] - ts.task_begin[p];
    // beta = 0: rows without entries become zeros; many of them go to the fill kernel below
    int64_t n_zero = (beta == 0.f) ? ntasks - ts.cnt_nonempty[(size_t)p] : 0;
    {
      int zvw, zlanes, zrows;
      if (n_zero < kZeroRowsWorthALaunch || !zero_rows_shape(Y, ldy, F, &zvw, &zlanes, &zrows)) n_zero = 0;
    }
    ntasks -= n_zero;
    BinTable& bt = a.bins;
    bt.n_bins = 0;
    bt.block_begin[0] = 0;
    bt.task_begin[0] = 0;
    int64_t begin = 0;
    for (int i = top; i >= 0; --i) {
      const int64_t end = (i == 0) ? ntasks : ts.cnt_ge[p][i];  // length >= 8 << i  => 1 << i lane groups
      if (end > begin) {
        bt.gpt_log2[bt.n_bins] = i;
        bt.block_begin[bt.n_bins + 1] = bt.block_begin[bt.n_bins] + spmm_bin_blocks(end - begin, lpr, i, n_chunks);
        bt.task_begin[bt.n_bins + 1] = end;
        ++bt.n_bins;
        begin = end;
      }
    }
    a.tasks = ts.d_tasks + ts.task_begin[p];
    if (bt.n_bins > 0) {
      const int rc = launch(vw, lpr, a);
      if (rc) return rc;
    }
    if (n_zero > 0) {
      const int rc = launch_zero_rows(a.tasks + ntasks, n_zero, F, Y, ldy, g->d_partial, g->ldp, a.stream);
      if (rc) return rc;
    }
    const int64_t nfix = ts.fix_begin[(size_t)p + 1] - ts.fix_begin[p];
    if (nfix > 0) {
      spmm_fixup<<<(unsigned)nfix, kThreads, 0, a.stream>>>(ts.d_fix + ts.fix_begin[p], nfix, g->d_partial,
                                                           g->ldp, F, beta, epilogue, Y, ldy);
      MGGCN_LAUNCH_CHECK();
    }
  }
  return MGGCN_OK;
}

}  // namespace

// Panel form and feature-slice width for one product.
// A wide operand on a graph with panel forms: when even the largest panel count leaves a panel
// of X well above the target size, the feature columns are walked in slices as well, one slice
// after the other (each costs one more pass over the entries, 8 bytes each, against a gather
// that then stays in the caches: F = 602 on the 233K-vertex graph measured 40 % faster).
const TaskSet& plan_passes(const mggcn_graph* g, const Orientation& o, int32_t F, int elem_bytes, int epilogue,
                           int64_t* slice_out) {
  const TaskSet& ts = *pick_panels(g, o, F, elem_bytes, epilogue);
  int64_t slice = std::max(F, 1);
  if (!g->panels_fixed && ts.n_panels > 1) {
    // Slices are cut for two thirds of the panel target: once the entries are walked several times
    // anyway, the smaller working set measured better (fp32 F=602: 17.6 -> 16.6 ms, F=256 7.2 -> 6.8 ms).
    const int64_t passes = ceil_div((int64_t)o.n_cols * F * elem_bytes, std::max<int64_t>(panel_target(g, elem_bytes) / 3 * 2, 1));
    if (passes > ts.n_panels) {
      // slices of whole 64-element groups keep every alignment of the full operand; a slice narrower
      // than 512 bytes of a row gathers too little per entry to pay for re-reading the entries
      slice = (int64_t)align_up((size_t)ceil_div(F, ceil_div(passes, ts.n_panels)), 64);
      slice = std::max<int64_t>(slice, 512 / elem_bytes);
    }
  }
  *slice_out = slice;
  return ts;
}

int spmm_run(const mggcn_graph* g, const Orientation& o, const void* X, int64_t ldx, int elem_bytes, int vw,
             int32_t F, float beta, int epilogue, float* Y, int64_t ldy, void* stream, SpmmLaunchFn launch) {
  int64_t slice = F;
  const TaskSet& ts = plan_passes(g, o, F, elem_bytes, epilogue, &slice);
  for (int64_t f = 0; f < F; f += slice) {
    const int rc = spmm_run_slice(g, o, ts, static_cast<const char*>(X) + f * elem_bytes, ldx, vw,
                                  (int32_t)std::min<int64_t>(slice, F - f), beta, epilogue, Y + f, ldy, stream, launch);
    if (rc) return rc;
  }
  return MGGCN_OK;
}

}  // namespace mggcn

using namespace mggcn;

extern "C" {

int mggcn_graph_create(int32_t n_rows, int32_t n_cols, const int32_t* rowptr, const int32_t* colidx,
                       const float* val, const int32_t* rowptr_t, const int32_t* colidx_t,
                       const float* val_t, int32_t seg_len, int32_t n_panels, void* stream,
                       mggcn_graph** out) {
  return graph_create_impl<int32_t>(n_rows, n_cols, rowptr, colidx, val, rowptr_t, colidx_t, val_t, seg_len,
                                    n_panels, stream, out);
}

int mggcn_graph_create64(int32_t n_rows, int32_t n_cols, const int64_t* rowptr, const int32_t* colidx,
                         const float* val, const int64_t* rowptr_t, const int32_t* colidx_t,
                         const float* val_t, int32_t seg_len, int32_t n_panels, void* stream,
                         mggcn_graph** out) {
  return graph_create_impl<int64_t>(n_rows, n_cols, rowptr, colidx, val, rowptr_t, colidx_t, val_t, seg_len,
                                    n_panels, stream, out);
}

size_t mggcn_graph_workspace_bytes(const mggcn_graph* g, int32_t F_max) {
  if (!g || F_max < 0) return 0;
  size_t bytes = 0;
  const int rc = guarded([&] { bytes = carve_graph(g, F_max, nullptr, nullptr); return (int)MGGCN_OK; });
  return rc ? 0 : bytes;
}

int mggcn_graph_bind(mggcn_graph* g, int32_t F_max, void* ws, size_t ws_bytes, void* stream) {
  MGGCN_REQUIRE(g != nullptr, MGGCN_E_INVALID_ARG, "graph is NULL");
  MGGCN_REQUIRE(F_max >= 1, MGGCN_E_INVALID_ARG, "F_max = %d must be positive", F_max);
  MGGCN_REQUIRE(ws && aligned(ws, kWsAlign), MGGCN_E_WORKSPACE, "workspace is NULL or not 256-byte aligned");
  const size_t need = mggcn_graph_workspace_bytes(g, F_max);
  MGGCN_REQUIRE(need > 0, MGGCN_E_NO_MEMORY, "out of host memory while sizing the workspace");
  MGGCN_REQUIRE(ws_bytes >= need, MGGCN_E_WORKSPACE, "workspace too small: %zu bytes given, %zu needed",
                ws_bytes, need);
  hipStream_t s = as_stream(stream);
  return guarded([&]() -> int {
    GraphCarve gc;
    carve_graph(g, F_max, ws, &gc);
    Orientation* os[2] = {&g->fwd, g->symmetric ? nullptr : &g->bwd};
    for (int o = 0; o < 2; ++o) {
      if (!os[o]) continue;
      const int rc = os[o]->wide ? build_tables<int64_t>(g, os[o], gc, o, s) : build_tables<int32_t>(g, os[o], gc, o, s);
      if (rc) return rc;
    }
    MGGCN_HIP(hipStreamSynchronize(s));
    g->d_partial = gc.partial;
    g->ldp = gc.ldp;
    g->F_bound = F_max;
    g->bound = true;
    return MGGCN_OK;
  });
}

int mggcn_graph_destroy(mggcn_graph* g) {
  delete g;
  return MGGCN_OK;
}

int mggcn_graph_tables(const mggcn_graph* g, int op, int32_t form, int32_t* n_panels, int64_t* n_tasks,
                       const void** tasks, int64_t* task_begin, int64_t* n_fix, const void** fix, int64_t* fix_begin,
                       int64_t* n_slots) {
  MGGCN_REQUIRE(g != nullptr, MGGCN_E_INVALID_ARG, "graph is NULL");
  MGGCN_REQUIRE(op == MGGCN_OP_N || op == MGGCN_OP_T, MGGCN_E_INVALID_ARG, "unknown op %d", op);
  MGGCN_REQUIRE(g->bound, MGGCN_E_WORKSPACE, "graph is not bound to a workspace");
  const Orientation& o = (op == MGGCN_OP_N || g->symmetric) ? g->fwd : g->bwd;
  MGGCN_REQUIRE(form >= 0 && form <= (int32_t)o.panelled.size(), MGGCN_E_INVALID_ARG, "form %d outside [0, %d]", form,
                (int)o.panelled.size());
  const TaskSet& ts = form == 0 ? o.flat : o.panelled[(size_t)form - 1];
  if (n_panels) *n_panels = ts.n_panels;
  if (n_tasks) *n_tasks = ts.task_begin[(size_t)ts.n_panels];
  if (tasks) *tasks = ts.d_tasks;
  if (n_fix) *n_fix = ts.fix_begin[(size_t)ts.n_panels];
  if (fix) *fix = ts.d_fix;
  if (n_slots) *n_slots = ts.n_slots;
  for (int32_t p = 0; p <= ts.n_panels; ++p) {
    if (task_begin) task_begin[p] = ts.task_begin[(size_t)p];
    if (fix_begin) fix_begin[p] = ts.fix_begin[(size_t)p];
  }
  return (int)o.panelled.size();
}

int mggcn_graph_tune(mggcn_graph* g, int32_t panel_mib, int32_t chunk_lanes) {
  MGGCN_REQUIRE(g != nullptr, MGGCN_E_INVALID_ARG, "graph is NULL");
  MGGCN_REQUIRE(panel_mib >= 0 && panel_mib <= (1 << 20), MGGCN_E_INVALID_ARG, "panel_mib %d outside [0, 2^20]",
                panel_mib);
  const bool lanes_ok = chunk_lanes == -1 || chunk_lanes == 0 ||
                        (chunk_lanes >= 1 && chunk_lanes <= 64 && (chunk_lanes & (chunk_lanes - 1)) == 0);
  MGGCN_REQUIRE(lanes_ok, MGGCN_E_INVALID_ARG, "chunk_lanes %d is not -1, 0 or a power of two up to 64", chunk_lanes);
  if (panel_mib > 0) g->panel_bytes = (int64_t)panel_mib << 20;
  if (chunk_lanes == -1) g->chunk_lanes = 0;
  else if (chunk_lanes > 0) g->chunk_lanes = chunk_lanes;
  return MGGCN_OK;
}

int mggcn_graph_panels(const mggcn_graph* g, int op, int32_t F) {
  MGGCN_REQUIRE(g != nullptr, MGGCN_E_INVALID_ARG, "graph is NULL");
  MGGCN_REQUIRE(op == MGGCN_OP_N || op == MGGCN_OP_T, MGGCN_E_INVALID_ARG, "unknown op %d", op);
  MGGCN_REQUIRE(F >= 0, MGGCN_E_INVALID_ARG, "F = %d is negative", F);
  const Orientation& o = (op == MGGCN_OP_N || g->symmetric) ? g->fwd : g->bwd;
  int64_t slice = F;
  const TaskSet& ts = plan_passes(g, o, F, (int)sizeof(float), MGGCN_EPI_NONE, &slice);
  return (int)(ts.n_panels * ceil_div(std::max(F, 1), slice));
}

int mggcn_spmm(const mggcn_graph* g, int op, const float* X, int64_t ldx, int32_t F, float beta,
               int epilogue, float* Y, int64_t ldy, void* stream) {
  int rc = spmm_check_args(g, op, X, ldx, (int)sizeof(float), F, beta, epilogue, Y, ldy);
  if (rc) return rc;
  const Orientation& o = (op == MGGCN_OP_N || g->symmetric) ? g->fwd : g->bwd;
  if (F == 0 || o.n_rows == 0) return MGGCN_OK;

  int vw = 1;
  if (aligned(X, 16) && aligned(Y, 16) && ldx % 4 == 0 && ldy % 4 == 0) vw = 4;
  else if (aligned(X, 8) && aligned(Y, 8) && ldx % 2 == 0 && ldy % 2 == 0) vw = 2;

  return spmm_run(g, o, X, ldx, (int)sizeof(float), vw, F, beta, epilogue, Y, ldy, stream, launch_any_f32);
}

}  // extern "C"
