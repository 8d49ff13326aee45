// Explicit CSR transpose on the device.  The backward SpMM of Eq. 9 runs on the transposed
// operator; for a non-symmetric A^ (the paper's in-degree-mean normalisation, or a rectangular
// row block) that needs A^^T as its own CSR.
//
// A stable radix sort of the entry positions by column index (rocPRIM through hipCUB -- setup
// code, not the hot path) yields, for every column, its entries in ascending row order, which
// is exactly the transposed CSR with ascending columns.  The result is unique, hence
// reproducible bit for bit.
#include "common.h"

#include <hipcub/hipcub.hpp>

namespace mggcn {
namespace {

constexpr int kThreads = 256;

__global__ __launch_bounds__(kThreads) void iota_i32(int64_t n, int32_t* out) {
  const int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (k < n) out[k] = (int32_t)k;
}

__global__ __launch_bounds__(kThreads) void zero_counts(int64_t n, int32_t* out) {
  const int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (k < n) out[k] = 0;
}

// integer histogram; an index outside [0, n_cols) (malformed input) is left out rather than followed
__global__ __launch_bounds__(kThreads) void count_columns(int64_t nnz, int32_t n_cols,
                                                           const int32_t* __restrict__ colidx,
                                                           int32_t* __restrict__ counts) {
  const int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (k < nnz && (uint32_t)colidx[k] < (uint32_t)n_cols) atomicAdd(&counts[colidx[k]], 1);
}

// pos[p] = original position of the p-th entry in column-major order
__global__ __launch_bounds__(kThreads) void gather_transposed(int64_t nnz, int32_t n_rows,
                                                               const int32_t* __restrict__ rowptr,
                                                               const float* __restrict__ val,
                                                               const int32_t* __restrict__ pos,
                                                               int32_t* __restrict__ colidx_t,
                                                               float* __restrict__ val_t) {
  const int64_t p = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (p >= nnz) return;
  const int32_t k = pos[p];
  // row of entry k: last i with rowptr[i] <= k
  int lo = 0, hi = n_rows;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (rowptr[mid + 1] <= k) lo = mid + 1; else hi = mid;
  }
  colidx_t[p] = lo;
  val_t[p] = val[k];
}

struct TWs {
  int32_t* counts;
  int32_t* scan_tmp;
  int32_t* keys_out;
  int32_t* pos_in;
  int32_t* pos_out;
  void* sort_tmp;
  size_t sort_tmp_bytes;
};

int end_bit_for(int32_t n_cols) {
  int b = 1;
  while (b < 31 && ((int64_t)1 << b) < (int64_t)n_cols) ++b;
  return b;
}

size_t carve(int32_t n_rows, int32_t n_cols, int64_t nnz, void* ws, TWs* out) {
  (void)n_rows;
  Carver c(ws);
  TWs w;
  w.counts = c.take<int32_t>((size_t)n_cols + 1);
  w.scan_tmp = c.take<int32_t>(scan_tmp_ints(n_cols));
  w.keys_out = c.take<int32_t>((size_t)nnz);
  w.pos_in = c.take<int32_t>((size_t)nnz);
  w.pos_out = c.take<int32_t>((size_t)nnz);
  size_t tmp = 0;
  // size query only: with a null temporary pointer nothing is launched
  const hipError_t qe = hipcub::DeviceRadixSort::SortPairs(
      nullptr, tmp, (const int32_t*)nullptr, (int32_t*)nullptr, (const int32_t*)nullptr,
      (int32_t*)nullptr, nnz, 0, end_bit_for(n_cols), (hipStream_t)0);
  if (qe != hipSuccess) tmp = (size_t)nnz * 16 + (1u << 20);  // no device to ask: generous bound
  w.sort_tmp_bytes = tmp;
  w.sort_tmp = c.take<char>(tmp + kWsAlign);
  if (out) *out = w;
  return c.off;
}

}  // namespace
}  // namespace mggcn

using namespace mggcn;

extern "C" {

size_t mggcn_csr_transpose_workspace_bytes(int32_t n_rows, int32_t n_cols, int64_t nnz) {
  if (n_rows < 0 || n_cols < 0 || nnz < 0 || nnz >= INT32_MAX) return 0;
  return carve(n_rows, n_cols, nnz, nullptr, nullptr);
}

int mggcn_csr_transpose(int32_t n_rows, int32_t n_cols, int64_t nnz, const int32_t* rowptr,
                        const int32_t* colidx, const float* val, int32_t* rowptr_t,
                        int32_t* colidx_t, float* val_t, void* ws, size_t ws_bytes, void* stream) {
  MGGCN_REQUIRE(n_rows >= 0 && n_cols >= 0 && nnz >= 0, MGGCN_E_INVALID_ARG,
                "negative size (%d x %d, nnz %lld)", n_rows, n_cols, (long long)nnz);
  MGGCN_REQUIRE(nnz < INT32_MAX, MGGCN_E_OVERFLOW, "nnz %lld does not fit int32", (long long)nnz);
  MGGCN_REQUIRE(rowptr && rowptr_t, MGGCN_E_INVALID_ARG, "rowptr / rowptr_t is NULL");
  MGGCN_REQUIRE(nnz == 0 || (colidx && val && colidx_t && val_t), MGGCN_E_INVALID_ARG,
                "colidx / val / colidx_t / val_t is NULL");
  MGGCN_REQUIRE(ws && aligned(ws, kWsAlign), MGGCN_E_WORKSPACE,
                "workspace is NULL or not 256-byte aligned");
  TWs w;
  const size_t need = carve(n_rows, n_cols, nnz, ws, &w);
  MGGCN_REQUIRE(ws_bytes >= need, MGGCN_E_WORKSPACE, "workspace too small: %zu bytes given, %zu needed",
                ws_bytes, need);
  hipStream_t s = as_stream(stream);
  zero_counts<<<(unsigned)ceil_div((int64_t)n_cols + 1, kThreads), kThreads, 0, s>>>((int64_t)n_cols + 1,
                                                                                    w.counts);
  MGGCN_LAUNCH_CHECK();
  if (nnz > 0) {
    const unsigned nb = (unsigned)ceil_div(nnz, kThreads);
    count_columns<<<nb, kThreads, 0, s>>>(nnz, n_cols, colidx, w.counts);
    MGGCN_LAUNCH_CHECK();
    iota_i32<<<nb, kThreads, 0, s>>>(nnz, w.pos_in);
    MGGCN_LAUNCH_CHECK();
  }
  int rc = exclusive_scan_i32(w.counts, n_cols, rowptr_t, w.scan_tmp, s);
  if (rc) return rc;
  if (nnz > 0) {
    size_t tmp = w.sort_tmp_bytes;
    MGGCN_HIP(hipcub::DeviceRadixSort::SortPairs(w.sort_tmp, tmp, colidx, w.keys_out, w.pos_in,
                                                 w.pos_out, nnz, 0, end_bit_for(n_cols), s));
    gather_transposed<<<(unsigned)ceil_div(nnz, kThreads), kThreads, 0, s>>>(
        nnz, n_rows, rowptr, val, w.pos_out, colidx_t, val_t);
    MGGCN_LAUNCH_CHECK();
  }
  return MGGCN_OK;
}

}  // extern "C"
