// Device-side construction of the SpMM's row-segment tables (see graph.h and spmm.hip for what they
// are): count -> prefix sums -> stable sort by (panel, length descending) -> fill.
//
// The definition, per row i of a matrix whose columns are cut into P equal panels: the entries of the
// row fall into at most P contiguous ranges (columns ascend inside a row); an empty row counts as one
// empty range in panel 0.  A range of at most seg_len entries is one task; a longer one is cut into
// ceil(len / seg_len) pieces of equal size (the last may be shorter), each a task that writes a
// partial sum ("slot"), and the range gets a fix-up record.  The first and the last range of a row
// carry the flags that tell a launch whether the caller's beta applies and whether the epilogue does.
// Tasks are listed panel after panel, inside a panel longest first, and in (row, piece) order among
// equal lengths -- so one launch per panel can bin its tasks by length as contiguous ranges, and the
// result does not depend on anything but the matrix.
//
// Steps (q = p * n_rows + i numbers the (panel, row) pairs panel-major, so that prefix sums over q
// give panel-major positions directly):
//   count_ranges   tasks / fix-up records / slots of every q
//   (three prefix sums)
//   range_keys     key of every task in generation order: p * (seg_len + 1) + (seg_len - length)
//   (stable radix sort of the keys, carrying the generation index)
//   fill_tasks     the task at each sorted position, recomputed from its generation index
//   fill_fix       the fix-up records, in generation order
//   summarise      per panel: first task, first fix-up record, slots, tasks at least 8 << k long
#include "common.h"
#include "graph.h"

#include <vector>

namespace mggcn {
namespace {

constexpr int kThreads = 256;

struct RowRange {
  int64_t lo;      // first entry
  int32_t len;     // entries
  uint32_t flags;  // kTaskFirst / kTaskLast
  bool present;    // the (row, panel) pair has a range
};

// The range of row i in panel p of P.  cuts: per row `stride` entry offsets at the boundaries of the
// finest panel width, of which every `step`-th is a boundary of this table's panels (unused for P = 1).
template <typename IT>
__device__ inline RowRange row_range(const IT* __restrict__ rowptr, const uint32_t* __restrict__ cuts, int stride, int step,
                                     int P, int64_t i, int p) {
  auto cut = [&](int c) -> int64_t {
    if (c == 0) return (int64_t)rowptr[i];
    if (c == P) return (int64_t)rowptr[i + 1];
    return (int64_t)cuts[i * stride + (int64_t)c * step - 1];
  };
  int first = -1, last = -1;
  int64_t prev = cut(0), lo = 0, hi = 0;
  for (int c = 0; c < P; ++c) {
    const int64_t next = cut(c + 1);
    if (next > prev) { if (first < 0) first = c; last = c; }
    if (c == p) { lo = prev; hi = next; }
    prev = next;
  }
  if (first < 0) first = last = 0;  // empty row: one empty range that still writes beta * Y / zeros
  RowRange r;
  r.lo = lo;
  r.len = (int32_t)(hi - lo);
  r.flags = (p == first ? kTaskFirst : 0u) | (p == last ? kTaskLast : 0u);
  r.present = p >= first && p <= last && !(r.len == 0 && !(p == first && first == last));
  return r;
}

__device__ inline int32_t pieces_of(int32_t len, int32_t seg_len) { return (len + seg_len - 1) / seg_len; }

template <typename IT>
__global__ __launch_bounds__(kThreads) void count_ranges(int64_t n_rows, int P, int seg_len, const IT* __restrict__ rowptr,
                                                          const uint32_t* __restrict__ cuts, int stride, int step,
                                                          int32_t* __restrict__ n_task, int32_t* __restrict__ n_fix,
                                                          int32_t* __restrict__ n_slot) {
  const int64_t q = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (q >= n_rows * P) return;
  const int p = (int)(q / n_rows);
  const int64_t i = q % n_rows;
  const RowRange r = row_range<IT>(rowptr, cuts, stride, step, P, i, p);
  int32_t t = 0, f = 0, s = 0;
  if (r.present) {
    if (r.len <= seg_len) t = 1;
    else { t = pieces_of(r.len, seg_len); f = 1; s = t; }
  }
  n_task[q] = t;
  n_fix[q] = f;
  n_slot[q] = s;
}

template <typename IT>
__global__ __launch_bounds__(kThreads) void range_keys(int64_t n_rows, int P, int seg_len, const IT* __restrict__ rowptr,
                                                        const uint32_t* __restrict__ cuts, int stride, int step,
                                                        const int64_t* __restrict__ task_off, uint32_t* __restrict__ keys) {
  const int64_t q = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (q >= n_rows * P) return;
  const int64_t begin = task_off[q], count = task_off[q + 1] - begin;
  if (count == 0) return;
  const int p = (int)(q / n_rows);
  const RowRange r = row_range<IT>(rowptr, cuts, stride, step, P, q % n_rows, p);
  const uint32_t base = (uint32_t)p * (uint32_t)(seg_len + 1);
  if (count == 1) { keys[begin] = base + (uint32_t)(seg_len - r.len); return; }
  const int32_t nseg = (int32_t)count, piece = (r.len + nseg - 1) / nseg;
  for (int32_t s = 0; s < nseg; ++s) {
    const int64_t k0 = (int64_t)s * piece;
    const int32_t len = (int32_t)max((int64_t)0, min((int64_t)r.len, k0 + piece) - k0);
    keys[begin + s] = base + (uint32_t)(seg_len - len);
  }
}

// order[pos] = generation index of the task that the stable sort put at position pos
template <typename IT>
__global__ __launch_bounds__(kThreads) void fill_tasks(int64_t n_tasks, int64_t n_rows, int P, int seg_len,
                                                        const IT* __restrict__ rowptr, const uint32_t* __restrict__ cuts,
                                                        int stride, int step, const int64_t* __restrict__ task_off,
                                                        const int64_t* __restrict__ slot_off,
                                                        const uint32_t* __restrict__ order, Task* __restrict__ tasks) {
  const int64_t pos = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (pos >= n_tasks) return;
  const int64_t u = order[pos];
  // the (panel, row) pair whose tasks hold generation index u: last q with task_off[q] <= u
  int64_t lo = 0, hi = n_rows * P;
  while (lo < hi) {
    const int64_t mid = (lo + hi) >> 1;
    if (task_off[mid + 1] <= u) lo = mid + 1; else hi = mid;
  }
  const int64_t q = lo;
  const int p = (int)(q / n_rows);
  const int64_t i = q % n_rows;
  const RowRange r = row_range<IT>(rowptr, cuts, stride, step, P, i, p);
  Task t;
  t.row = (int32_t)i;
  if (r.len <= seg_len) {
    t.k0 = (uint32_t)r.lo;
    t.len_flags = (uint32_t)r.len | r.flags;
    t.slot = -1;
  } else {
    const int32_t nseg = pieces_of(r.len, seg_len), piece = (r.len + nseg - 1) / nseg;
    const int32_t s = (int32_t)(u - task_off[q]);
    const int64_t k0 = (int64_t)s * piece;
    t.k0 = (uint32_t)(r.lo + k0);
    t.len_flags = (uint32_t)max((int64_t)0, min((int64_t)r.len, k0 + piece) - k0);  // pieces carry no flags
    t.slot = (int32_t)(slot_off[q] - slot_off[(int64_t)p * n_rows]) + s;     // slots are numbered per panel
  }
  tasks[pos] = t;
}

template <typename IT>
__global__ __launch_bounds__(kThreads) void fill_fix(int64_t n_rows, int P, int seg_len, const IT* __restrict__ rowptr,
                                                      const uint32_t* __restrict__ cuts, int stride, int step,
                                                      const int64_t* __restrict__ fix_off, const int64_t* __restrict__ slot_off,
                                                      FixRow* __restrict__ fix) {
  const int64_t q = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (q >= n_rows * P) return;
  if (fix_off[q + 1] == fix_off[q]) return;
  const int p = (int)(q / n_rows);
  const int64_t i = q % n_rows;
  const RowRange r = row_range<IT>(rowptr, cuts, stride, step, P, i, p);
  FixRow f;
  f.row = (int32_t)i;
  f.slot0 = (int32_t)(slot_off[q] - slot_off[(int64_t)p * n_rows]);
  f.nslots = pieces_of(r.len, seg_len);
  f.flags = r.flags;
  fix[fix_off[q]] = f;
}

// out[p * kSummary + ...]: first task, first fix-up record, slots of panel p, then for k = 0..6 the number of its
// tasks at least 8 << k long (keys ascend: longest first); entry P holds the totals.
constexpr int kSummary = 3 + kLenClasses + 1;  // the last one: tasks with at least one entry
__global__ void summarise(int64_t n_rows, int P, int seg_len, const int64_t* __restrict__ task_off,
                          const int64_t* __restrict__ fix_off, const int64_t* __restrict__ slot_off,
                          const uint32_t* __restrict__ sorted_keys, int64_t* __restrict__ out) {
  const int p = blockIdx.x, k = threadIdx.x;  // P + 1 blocks of kSummary threads
  const int64_t q0 = (int64_t)p * n_rows;
  const int64_t t0 = task_off[q0];
  if (k == 0) out[p * kSummary + 0] = t0;
  if (k == 1) out[p * kSummary + 1] = fix_off[q0];
  if (k == 2) out[p * kSummary + 2] = p < P ? slot_off[q0 + n_rows] - slot_off[q0] : 0;
  if (k >= 3 && p < P) {
    const int32_t len = k < 3 + kLenClasses ? 8 << (k - 3) : 1;
    int64_t n = 0;
    if (len <= seg_len) {  // tasks of panel p with key <= p * (seg_len + 1) + (seg_len - len)
      const uint32_t bound = (uint32_t)p * (uint32_t)(seg_len + 1) + (uint32_t)(seg_len - len);
      int64_t lo = t0, hi = task_off[q0 + n_rows];
      while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (sorted_keys[mid] <= bound) lo = mid + 1; else hi = mid;
      }
      n = lo - t0;
    }
    out[p * kSummary + k] = n;
  }
  if (k >= 3 && p == P) out[p * kSummary + k] = 0;
}

struct BuildCarve {
  int32_t *n_task, *n_fix, *n_slot;
  int64_t *task_off, *fix_off, *slot_off, *scan_tmp, *summary;
  uint32_t *keys, *keys_sorted, *order;
  void* sort_tmp;
};

size_t carve_build(int64_t n_rows, int32_t P, int64_t max_tasks, void* scratch, BuildCarve* out) {
  const size_t Q = (size_t)std::max<int64_t>(n_rows, 1) * (size_t)P;
  const size_t T = (size_t)std::max<int64_t>(max_tasks, 1);
  Carver c(scratch);
  BuildCarve w;
  w.n_task = c.take<int32_t>(Q);
  w.n_fix = c.take<int32_t>(Q);
  w.n_slot = c.take<int32_t>(Q);
  w.task_off = c.take<int64_t>(Q + 1);
  w.fix_off = c.take<int64_t>(Q + 1);
  w.slot_off = c.take<int64_t>(Q + 1);
  w.scan_tmp = c.take<int64_t>(scan_tmp_ints((int64_t)Q));
  w.summary = c.take<int64_t>((size_t)(P + 1) * kSummary);
  w.keys = c.take<uint32_t>(T);
  w.keys_sorted = c.take<uint32_t>(T);
  w.order = c.take<uint32_t>(T);
  w.sort_tmp = c.take<char>(radix_sort_tmp_bytes((int64_t)T));
  if (out) *out = w;
  return c.off;
}

int key_bits_for(int64_t n_keys) {
  int b = 1;
  while (b < 32 && ((int64_t)1 << b) < n_keys) ++b;
  return b;
}

}  // namespace

size_t task_build_scratch_bytes(int64_t n_rows, int32_t n_panels, int64_t max_tasks) {
  return carve_build(n_rows, std::max(n_panels, 1), max_tasks, nullptr, nullptr);
}

template <typename IT>
int build_task_set_device(TaskSet* ts, int64_t n_rows, const IT* rowptr, const uint32_t* cuts, int32_t cut_stride,
                          int32_t cut_step, int32_t seg_len, Task* d_tasks, FixRow* d_fix, void* scratch, hipStream_t s) {
  const int32_t P = std::max(ts->n_panels, 1);
  ts->task_begin.assign((size_t)P + 1, 0);
  ts->fix_begin.assign((size_t)P + 1, 0);
  ts->cnt_ge.assign((size_t)P, {});
  ts->cnt_nonempty.assign((size_t)P, 0);
  ts->n_slots = 0;
  ts->d_tasks = d_tasks;
  ts->d_fix = d_fix;
  if (n_rows <= 0) return MGGCN_OK;
  BuildCarve w;
  carve_build(n_rows, P, ts->max_tasks, scratch, &w);
  const int64_t Q = n_rows * P;
  MGGCN_REQUIRE(ceil_div(Q, kThreads) < ((int64_t)1 << 31), MGGCN_E_OVERFLOW, "%lld (row, panel) pairs: grid too large",
                (long long)Q);
  const unsigned qb = (unsigned)ceil_div(Q, kThreads);
  count_ranges<IT><<<qb, kThreads, 0, s>>>(n_rows, P, seg_len, rowptr, cuts, cut_stride, cut_step, w.n_task, w.n_fix, w.n_slot);
  MGGCN_LAUNCH_CHECK();
  int rc = exclusive_scan_i64(w.n_task, Q, w.task_off, w.scan_tmp, s);
  if (!rc) rc = exclusive_scan_i64(w.n_fix, Q, w.fix_off, w.scan_tmp, s);
  if (!rc) rc = exclusive_scan_i64(w.n_slot, Q, w.slot_off, w.scan_tmp, s);
  if (rc) return rc;
  // the totals decide the launches below; they also check the host's upper bounds
  int64_t totals[3] = {0, 0, 0};
  MGGCN_HIP(hipMemcpyAsync(&totals[0], w.task_off + Q, sizeof(int64_t), hipMemcpyDeviceToHost, s));
  MGGCN_HIP(hipMemcpyAsync(&totals[1], w.fix_off + Q, sizeof(int64_t), hipMemcpyDeviceToHost, s));
  MGGCN_HIP(hipMemcpyAsync(&totals[2], w.slot_off + Q, sizeof(int64_t), hipMemcpyDeviceToHost, s));
  MGGCN_HIP(hipStreamSynchronize(s));
  const int64_t T = totals[0];
  MGGCN_REQUIRE(T <= ts->max_tasks && totals[1] <= ts->max_fix && totals[2] <= ts->max_slots, MGGCN_E_WORKSPACE,
                "segment tables need %lld tasks / %lld fix-up rows / %lld slots, sized for %lld / %lld / %lld",
                (long long)T, (long long)totals[1], (long long)totals[2], (long long)ts->max_tasks, (long long)ts->max_fix,
                (long long)ts->max_slots);
  MGGCN_REQUIRE(T < ((int64_t)1 << 32), MGGCN_E_OVERFLOW, "%lld tasks: positions are held in 32 unsigned bits", (long long)T);
  if (T > 0) {
    range_keys<IT><<<qb, kThreads, 0, s>>>(n_rows, P, seg_len, rowptr, cuts, cut_stride, cut_step, w.task_off, w.keys);
    MGGCN_LAUNCH_CHECK();
    rc = radix_sort_pairs(w.keys, nullptr, w.keys_sorted, w.order, T, key_bits_for((int64_t)P * (seg_len + 1)), w.sort_tmp, s);
    if (rc) return rc;
    fill_tasks<IT><<<(unsigned)ceil_div(T, kThreads), kThreads, 0, s>>>(T, n_rows, P, seg_len, rowptr, cuts, cut_stride, cut_step,
                                                                        w.task_off, w.slot_off, w.order, d_tasks);
    MGGCN_LAUNCH_CHECK();
  }
  if (totals[1] > 0) {
    fill_fix<IT><<<qb, kThreads, 0, s>>>(n_rows, P, seg_len, rowptr, cuts, cut_stride, cut_step, w.fix_off, w.slot_off, d_fix);
    MGGCN_LAUNCH_CHECK();
  }
  summarise<<<P + 1, kSummary, 0, s>>>(n_rows, P, seg_len, w.task_off, w.fix_off, w.slot_off, w.keys_sorted, w.summary);
  MGGCN_LAUNCH_CHECK();
  std::vector<int64_t> sum((size_t)(P + 1) * kSummary);
  MGGCN_HIP(hipMemcpyAsync(sum.data(), w.summary, sizeof(int64_t) * sum.size(), hipMemcpyDeviceToHost, s));
  MGGCN_HIP(hipStreamSynchronize(s));
  for (int32_t p = 0; p <= P; ++p) {
    ts->task_begin[(size_t)p] = sum[(size_t)p * kSummary + 0];
    ts->fix_begin[(size_t)p] = sum[(size_t)p * kSummary + 1];
    if (p < P) {
      ts->n_slots = std::max(ts->n_slots, sum[(size_t)p * kSummary + 2]);
      for (int k = 0; k < kLenClasses; ++k) ts->cnt_ge[(size_t)p][(size_t)k] = sum[(size_t)p * kSummary + 3 + k];
      ts->cnt_nonempty[(size_t)p] = sum[(size_t)p * kSummary + 3 + kLenClasses];
    }
  }
  return MGGCN_OK;
}

template int build_task_set_device<int32_t>(TaskSet*, int64_t, const int32_t*, const uint32_t*, int32_t, int32_t, int32_t,
                                            Task*, FixRow*, void*, hipStream_t);
template int build_task_set_device<int64_t>(TaskSet*, int64_t, const int64_t*, const uint32_t*, int32_t, int32_t, int32_t,
                                            Task*, FixRow*, void*, hipStream_t);

}  // namespace mggcn
