// Host-side representation of a graph handle: the borrowed CSR arrays of A^ (and of A^^T when
// the operator is not symmetric) plus the row-segment tables the SpMM kernels walk.
#pragma once

#include <cstdint>
#include <vector>

namespace mggcn {

struct Task {
  int32_t row, k0, k1, slot;  // slot < 0: final result of the row; else index into partials
};
struct FixRow {
  int32_t row, slot0, nslots, pad;
};

constexpr int kLenClasses = 7;  // thresholds 8*2^i, i = 0..6

struct Orientation {
  int32_t n_rows = 0, n_cols = 0;
  int64_t nnz = 0;
  const int32_t* rowptr = nullptr;
  const int32_t* colidx = nullptr;
  const float* val = nullptr;
  std::vector<Task> tasks;
  std::vector<FixRow> fix;
  int64_t n_slots = 0;
  int64_t cnt_ge[kLenClasses] = {0};  // tasks with length >= 8 << i
  Task* d_tasks = nullptr;
  FixRow* d_fix = nullptr;
};

}  // namespace mggcn

struct mggcn_graph {
  mggcn::Orientation fwd, bwd;
  bool symmetric = true;
  int32_t seg_len = 0;
  int32_t F_bound = 0;
  int64_t ldp = 0;
  float* d_partial = nullptr;
  bool bound = false;
  int32_t chunk_lanes = 0;  // forced lanes per feature chunk (0 = widest)
};

