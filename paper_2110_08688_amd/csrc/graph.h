// Host-side representation of a graph handle: the borrowed CSR arrays of A^ (and of A^^T when
// the operator is not symmetric) plus the row-segment tables the SpMM kernels walk.
#pragma once

#include <hip/hip_runtime.h>

#include <array>
#include <cstdint>
#include <vector>

namespace mggcn {

// One unit of SpMM work: `len` consecutive entries of one row, starting at entry k0.
// len_flags packs the length with two flags:
//   first: no earlier launch has written this row, so the caller's beta applies (else beta = 1)
//   last : no later launch adds to this row, so the epilogue is applied here
struct Task {
  int32_t row;
  uint32_t k0;  // entry offsets are held in 32 unsigned bits: fewer than 2^32 entries per matrix
  uint32_t len_flags;
  int32_t slot;  // < 0: result goes to Y; else index into the partial-sum table
};
constexpr uint32_t kTaskFirst = 1u << 30, kTaskLast = 1u << 29, kTaskLenMask = (1u << 29) - 1;

// A (row, panel) range that was cut into several tasks: its partial sums are added in order.
struct FixRow {
  int32_t row, slot0, nslots;
  uint32_t flags;  // kTaskFirst / kTaskLast as above
};

constexpr int kLenClasses = 7;  // length thresholds 8 << i, i = 0..6

// Tasks of one operator, grouped by column panel (panel p holds the entries whose column lies
// in the p-th equal slice of the column range).  One panel = the classic row split.
struct TaskSet {
  int32_t n_panels = 0;  // 0: not built
  // upper bounds from the row lengths alone (known when the handle is created: they size the workspace)
  int64_t max_tasks = 0, max_fix = 0, max_slots = 0;
  // exact figures, known once the tables have been built on the device (mggcn_graph_bind)
  std::vector<int64_t> task_begin;  // n_panels + 1 offsets into the task list (panel-major; inside a panel longest first)
  std::vector<int64_t> fix_begin;   // n_panels + 1 offsets into the fix-up records
  std::vector<std::array<int64_t, kLenClasses>> cnt_ge;  // per panel: tasks of length >= 8 << i
  std::vector<int64_t> cnt_nonempty;  // per panel: tasks with at least one entry (the rest, all of them rows
                                      // without any entry, are the tail of the panel's task list, rows ascending)
  int64_t n_slots = 0;              // partial-sum rows needed by the widest panel
  Task* d_tasks = nullptr;
  FixRow* d_fix = nullptr;
};

struct Orientation {
  int32_t n_rows = 0, n_cols = 0;
  int64_t nnz = 0;
  const void* rowptr = nullptr;  // device array of n_rows + 1 offsets, int32_t or (wide) int64_t
  bool wide = false;
  const int32_t* colidx = nullptr;
  const float* val = nullptr;
  int32_t finest = 1;  // panel count of the finest panel table (1: none); the others use every 2nd, 4th, ... boundary
  TaskSet flat;      // one panel
  // Column-panel forms: either the one panel count the caller asked for, or one per power of two
  // up to what the average row length affords; a product picks by the size of its gathered operand.
  std::vector<TaskSet> panelled;
};

// tasks.hip: the tables of one TaskSet built on the device into d_tasks / d_fix (room for max_tasks + 1 /
// max_fix + 1 records); fills the exact figures of *ts; synchronises the stream.  cuts: per row
// `cut_stride` entry offsets at the finest panel boundaries (device; unused for one panel).
size_t task_build_scratch_bytes(int64_t n_rows, int32_t n_panels, int64_t max_tasks);
template <typename IT>
int build_task_set_device(TaskSet* ts, int64_t n_rows, const IT* rowptr, const uint32_t* cuts, int32_t cut_stride,
                          int32_t cut_step, int32_t seg_len, Task* d_tasks, FixRow* d_fix, void* scratch, hipStream_t s);

}  // namespace mggcn

struct mggcn_graph {
  mggcn::Orientation fwd, bwd;
  bool symmetric = true;
  int32_t seg_len = 0;
  int32_t F_bound = 0;
  int64_t ldp = 0;
  float* d_partial = nullptr;
  bool bound = false;
  int32_t chunk_lanes = 0;     // forced lanes per feature chunk (0 = widest)
  int64_t panel_bytes = 0;      // one column panel of the gathered operand should be about this large
  bool panels_fixed = false;    // the caller chose the panel count: use it whatever the operand size
};
