// Explicit CSR transpose on the device.  The backward SpMM of Eq. 9 runs on the transposed
// operator; for a non-symmetric A^ (the paper's in-degree-mean normalisation, or a rectangular
// row block) that needs A^^T as its own CSR.
//
// A counting sort by column in three steps, all of them this library's own kernels: an integer
// histogram of the column indices and its prefix sum give the row offsets of A^^T; a stable radix
// sort of the entry positions by column index (sort.hip) yields, for every column, its entries in
// ascending row order -- exactly the transposed CSR with ascending columns; a last pass looks up
// the row of every entry (binary search in the row offsets) and moves the values.  The result is
// unique, hence reproducible bit for bit.  Row offsets of 32 or 64 bits (fewer than 2^32 entries).
#include "common.h"

namespace mggcn {
namespace {

constexpr int kThreads = 256;

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
template <typename IT>
__global__ __launch_bounds__(kThreads) void gather_transposed(int64_t nnz, int32_t n_rows,
                                                               const IT* __restrict__ rowptr,
                                                               const float* __restrict__ val,
                                                               const uint32_t* __restrict__ pos,
                                                               int32_t* __restrict__ colidx_t,
                                                               float* __restrict__ val_t) {
  const int64_t p = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (p >= nnz) return;
  const int64_t k = pos[p];
  // row of entry k: last i with rowptr[i] <= k
  int lo = 0, hi = n_rows;
  while (lo < hi) {
    const int mid = (int)(((int64_t)lo + hi) >> 1);
    if ((int64_t)rowptr[mid + 1] <= k) lo = mid + 1; else hi = mid;
  }
  colidx_t[p] = lo;
  val_t[p] = val[k];
}

struct TWs {
  int32_t* counts;
  int64_t* scan_tmp;
  uint32_t* keys_out;
  uint32_t* pos_out;
  void* sort_tmp;
};

int key_bits_for(int32_t n_cols) {
  int b = 1;
  while (b < 31 && ((int64_t)1 << b) < (int64_t)n_cols) ++b;
  return b;
}

size_t carve(int32_t n_cols, int64_t nnz, void* ws, TWs* out) {
  Carver c(ws);
  TWs w;
  w.counts = c.take<int32_t>((size_t)n_cols + 1);
  w.scan_tmp = c.take<int64_t>(scan_tmp_ints(n_cols));  // sized for the 64-bit scan, serves the 32-bit one too
  w.keys_out = c.take<uint32_t>((size_t)std::max<int64_t>(nnz, 1));
  w.pos_out = c.take<uint32_t>((size_t)std::max<int64_t>(nnz, 1));
  w.sort_tmp = c.take<char>(radix_sort_tmp_bytes(nnz));
  if (out) *out = w;
  return c.off;
}

int scan_offsets(const int32_t* counts, int64_t n, int32_t* out, int64_t* tmp, hipStream_t s) {
  return exclusive_scan_i32(counts, n, out, reinterpret_cast<int32_t*>(tmp), s);
}
int scan_offsets(const int32_t* counts, int64_t n, int64_t* out, int64_t* tmp, hipStream_t s) {
  return exclusive_scan_i64(counts, n, out, tmp, s);
}

template <typename IT>
int transpose_impl(int32_t n_rows, int32_t n_cols, int64_t nnz, const IT* rowptr, const int32_t* colidx,
                   const float* val, IT* rowptr_t, int32_t* colidx_t, float* val_t, void* ws, size_t ws_bytes,
                   void* stream) {
  MGGCN_REQUIRE(n_rows >= 0 && n_cols >= 0 && nnz >= 0, MGGCN_E_INVALID_ARG,
                "negative size (%d x %d, nnz %lld)", n_rows, n_cols, (long long)nnz);
  if (sizeof(IT) == 4)
    MGGCN_REQUIRE(nnz < INT32_MAX, MGGCN_E_OVERFLOW, "nnz %lld does not fit 32-bit row offsets", (long long)nnz);
  MGGCN_REQUIRE(nnz < ((int64_t)1 << 32), MGGCN_E_OVERFLOW, "nnz %lld: entry positions are held in 32 unsigned bits",
                (long long)nnz);
  MGGCN_REQUIRE(rowptr && rowptr_t, MGGCN_E_INVALID_ARG, "rowptr / rowptr_t is NULL");
  MGGCN_REQUIRE(nnz == 0 || (colidx && val && colidx_t && val_t), MGGCN_E_INVALID_ARG,
                "colidx / val / colidx_t / val_t is NULL");
  MGGCN_REQUIRE(ws && aligned(ws, kWsAlign), MGGCN_E_WORKSPACE,
                "workspace is NULL or not 256-byte aligned");
  TWs w;
  const size_t need = carve(n_cols, nnz, ws, &w);
  MGGCN_REQUIRE(ws_bytes >= need, MGGCN_E_WORKSPACE, "workspace too small: %zu bytes given, %zu needed",
                ws_bytes, need);
  hipStream_t s = as_stream(stream);
  zero_counts<<<(unsigned)ceil_div((int64_t)n_cols + 1, kThreads), kThreads, 0, s>>>((int64_t)n_cols + 1,
                                                                                    w.counts);
  MGGCN_LAUNCH_CHECK();
  if (nnz > 0) {
    MGGCN_REQUIRE(ceil_div(nnz, kThreads) < ((int64_t)1 << 31), MGGCN_E_OVERFLOW, "grid too large");
    count_columns<<<(unsigned)ceil_div(nnz, kThreads), kThreads, 0, s>>>(nnz, n_cols, colidx, w.counts);
    MGGCN_LAUNCH_CHECK();
  }
  int rc = scan_offsets(w.counts, n_cols, rowptr_t, w.scan_tmp, s);
  if (rc) return rc;
  if (nnz > 0) {
    rc = radix_sort_pairs(reinterpret_cast<const uint32_t*>(colidx), nullptr, w.keys_out, w.pos_out, nnz,
                          key_bits_for(n_cols), w.sort_tmp, s);
    if (rc) return rc;
    gather_transposed<IT><<<(unsigned)ceil_div(nnz, kThreads), kThreads, 0, s>>>(nnz, n_rows, rowptr, val, w.pos_out,
                                                                                colidx_t, val_t);
    MGGCN_LAUNCH_CHECK();
  }
  return MGGCN_OK;
}

}  // namespace
}  // namespace mggcn

using namespace mggcn;

extern "C" {

size_t mggcn_csr_transpose_workspace_bytes(int32_t n_rows, int32_t n_cols, int64_t nnz) {
  if (n_rows < 0 || n_cols < 0 || nnz < 0 || nnz >= ((int64_t)1 << 32)) return 0;
  return carve(n_cols, nnz, nullptr, nullptr);
}

int mggcn_csr_transpose(int32_t n_rows, int32_t n_cols, int64_t nnz, const int32_t* rowptr,
                        const int32_t* colidx, const float* val, int32_t* rowptr_t,
                        int32_t* colidx_t, float* val_t, void* ws, size_t ws_bytes, void* stream) {
  return transpose_impl<int32_t>(n_rows, n_cols, nnz, rowptr, colidx, val, rowptr_t, colidx_t, val_t, ws, ws_bytes,
                                 stream);
}

int mggcn_csr_transpose64(int32_t n_rows, int32_t n_cols, int64_t nnz, const int64_t* rowptr,
                          const int32_t* colidx, const float* val, int64_t* rowptr_t,
                          int32_t* colidx_t, float* val_t, void* ws, size_t ws_bytes, void* stream) {
  return transpose_impl<int64_t>(n_rows, n_cols, nnz, rowptr, colidx, val, rowptr_t, colidx_t, val_t, ws, ws_bytes,
                                 stream);
}

}  // extern "C"
