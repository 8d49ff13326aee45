// Normalised adjacency A^ = D^-1/2 (A + I) D^-1/2 built on the device (Eq. 1-2 of the
// paper with Kipf-style self-loops), plus the paper's own in-degree-mean variant (Eq. 2).
//
// Three steps, all integer except the final value:
//   count : entries per row of A~ = A united with the diagonal (binary search for (i,i))
//   scan  : rowptr of A~
//   fill  : one wavefront per row copies the row, slots the diagonal in at its sorted
//           position and evaluates 1/sqrt(d_i d_j) in fp64, rounded once to fp32.
#include "common.h"

namespace mggcn {
namespace {

constexpr int kThreads = 256;

__device__ inline int lower_bound_dev(const int32_t* __restrict__ a, int n, int key) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (a[mid] < key) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// IT: type of the row offsets, int32_t or int64_t (entry counts beyond 2^31); a single row is
// always shorter than 2^31.
template <typename IT>
__global__ __launch_bounds__(kThreads) void count_rows(int32_t n_rows, int32_t n_cols,
                                                        const IT* __restrict__ rowptr,
                                                        const int32_t* __restrict__ colidx,
                                                        int32_t* __restrict__ counts) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= n_rows) return;
  const IT b = rowptr[i];
  const int32_t deg = (int32_t)(rowptr[i + 1] - b);
  int add = 0;
  if (i < n_cols) {
    const int p = lower_bound_dev(colidx + b, deg, (int)i);
    add = !(p < deg && colidx[b + p] == (int32_t)i);
  }
  counts[i] = deg + add;
}

// flag bit 0: rowptr not monotone / negative; bit 1: column out of range; bit 2: row not
// strictly ascending
template <typename IT>
__global__ __launch_bounds__(kThreads) void validate_rows(int32_t n_rows, int32_t n_cols,
                                                           const IT* __restrict__ rowptr,
                                                           const int32_t* __restrict__ colidx,
                                                           int64_t nnz, int32_t* flag) {
  const int lane = threadIdx.x & 63;
  const int64_t row = ((int64_t)blockIdx.x * kThreads + threadIdx.x) >> 6;
  if (row >= n_rows) return;
  const int64_t b = rowptr[row], e = rowptr[row + 1];
  int bad = 0;
  if (b < 0 || e < b || e > nnz || e - b > INT32_MAX) {
    bad = 1;
  } else {
    for (int64_t k = b + lane; k < e; k += 64) {
      const int32_t j = colidx[k];
      if (j < 0 || j >= n_cols) bad |= 2;
      if (k > b && colidx[k - 1] >= j) bad |= 4;
    }
  }
  if (bad) atomicOr(flag, bad);
}

// One wavefront per row.
template <bool kValues, typename IT>
__global__ __launch_bounds__(kThreads) void fill_rows(int32_t n_rows, int32_t n_cols,
                                                       const IT* __restrict__ rowptr_in,
                                                       const int32_t* __restrict__ colidx_in,
                                                       const int32_t* __restrict__ deg_row,
                                                       const int32_t* __restrict__ deg_col,
                                                       const IT* __restrict__ rowptr_out,
                                                       int32_t* __restrict__ colidx_out,
                                                       float* __restrict__ val_out) {
  const int lane = threadIdx.x & 63;
  const int64_t i = ((int64_t)blockIdx.x * kThreads + threadIdx.x) >> 6;
  if (i >= n_rows) return;
  const IT b = rowptr_in[i], ob = rowptr_out[i];
  const int32_t deg = (int32_t)(rowptr_in[i + 1] - b), odeg = (int32_t)(rowptr_out[i + 1] - ob);
  const bool insert = odeg != deg;  // the diagonal is missing from the input row
  const int p = insert ? lower_bound_dev(colidx_in + b, deg, (int)i) : 0;
  double di = 0.0;
  if (kValues) di = deg_row ? (double)deg_row[i] : (double)odeg;
  for (int32_t t = lane; t < odeg; t += 64) {
    int32_t j;
    if (insert && t == p) j = (int32_t)i;
    else j = colidx_in[b + t - ((insert && t > p) ? 1 : 0)];
    colidx_out[ob + t] = j;
    if (kValues) {
      const double dj = deg_col ? (double)deg_col[j] : (double)(rowptr_out[j + 1] - rowptr_out[j]);
      val_out[ob + t] = (float)(1.0 / sqrt(di * dj));
    }
  }
}

__global__ __launch_bounds__(kThreads) void column_histogram(int64_t nnz,
                                                              const int32_t* __restrict__ colidx,
                                                              int32_t* __restrict__ hist) {
  const int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (k < nnz) atomicAdd(&hist[colidx[k]], 1);  // integer counts: order-independent
}

__global__ __launch_bounds__(kThreads) void mean_values(int64_t nnz,
                                                         const int32_t* __restrict__ colidx,
                                                         const int32_t* __restrict__ colcount,
                                                         float* __restrict__ val) {
  const int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (k < nnz) val[k] = (float)(1.0 / (double)colcount[colidx[k]]);
}

__global__ void zero_i32(int32_t* p, int64_t n) {
  const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k < n) p[k] = 0;
}

struct NormWs {
  int32_t* counts;
  int32_t* scan_tmp;
  int32_t* colcount;
  int32_t* flag;
};

size_t carve(int32_t n_rows, int32_t n_cols, void* ws, NormWs* out) {
  Carver c(ws);
  NormWs w;
  w.counts = c.take<int32_t>((size_t)n_rows + 1);
  w.scan_tmp = c.take<int32_t>(2 * scan_tmp_ints(n_rows));  // room for 64-bit offsets
  w.colcount = c.take<int32_t>((size_t)n_cols + 1);
  w.flag = c.take<int32_t>(64);
  if (out) *out = w;
  return c.off;
}

int check_common(int32_t n_rows, int32_t n_cols, const void* rowptr_in, const void* colidx_in,
                 const void* ws, size_t ws_bytes) {
  MGGCN_REQUIRE(n_rows >= 0 && n_cols >= 0, MGGCN_E_INVALID_ARG, "negative matrix size %d x %d",
                n_rows, n_cols);
  MGGCN_REQUIRE(rowptr_in != nullptr, MGGCN_E_INVALID_ARG, "rowptr_in is NULL");
  (void)colidx_in;
  MGGCN_REQUIRE(ws != nullptr && aligned(ws, kWsAlign), MGGCN_E_WORKSPACE,
                "workspace is NULL or not 256-byte aligned");
  MGGCN_REQUIRE(ws_bytes >= carve(n_rows, n_cols, nullptr, nullptr), MGGCN_E_WORKSPACE,
                "workspace too small: %zu bytes given, %zu needed", ws_bytes,
                carve(n_rows, n_cols, nullptr, nullptr));
  return MGGCN_OK;
}

template <typename IT>
int normalize_count_impl(int32_t n_rows, int32_t n_cols, const IT* rowptr_in, const int32_t* colidx_in,
                         int validate, IT* rowptr_out, int64_t* nnz_out, void* ws, size_t ws_bytes,
                         void* stream) {
  int rc = check_common(n_rows, n_cols, rowptr_in, colidx_in, ws, ws_bytes);
  if (rc) return rc;
  MGGCN_REQUIRE(rowptr_out && nnz_out, MGGCN_E_INVALID_ARG, "rowptr_out / nnz_out is NULL");
  hipStream_t s = as_stream(stream);
  NormWs w;
  carve(n_rows, n_cols, ws, &w);

  IT nnz_in = 0;
  MGGCN_HIP(hipMemcpyAsync(&nnz_in, rowptr_in + n_rows, sizeof(IT), hipMemcpyDeviceToHost, s));
  MGGCN_HIP(hipStreamSynchronize(s));
  MGGCN_REQUIRE(nnz_in >= 0, MGGCN_E_BAD_CSR, "rowptr_in[n_rows] = %lld is negative", (long long)nnz_in);
  MGGCN_REQUIRE(nnz_in == 0 || colidx_in != nullptr, MGGCN_E_INVALID_ARG, "colidx_in is NULL");
  const int64_t worst = (int64_t)nnz_in + (n_rows < n_cols ? n_rows : n_cols);
  if (sizeof(IT) == 4)
    MGGCN_REQUIRE(worst < INT32_MAX, MGGCN_E_OVERFLOW,
                  "pattern with self-loops may reach %lld entries, int32 offsets hold 2^31-1: use the 64-bit form",
                  (long long)worst);
  else
    MGGCN_REQUIRE(worst < ((int64_t)1 << 32), MGGCN_E_OVERFLOW,
                  "pattern with self-loops may reach %lld entries, the library holds fewer than 2^32",
                  (long long)worst);

  if (validate) {
    zero_i32<<<1, 64, 0, s>>>(w.flag, 1);
    MGGCN_LAUNCH_CHECK();
    if (n_rows > 0) {
      validate_rows<IT><<<(unsigned)ceil_div((int64_t)n_rows * 64, kThreads), kThreads, 0, s>>>(
          n_rows, n_cols, rowptr_in, colidx_in, (int64_t)nnz_in, w.flag);
      MGGCN_LAUNCH_CHECK();
    }
    int32_t flag = 0;
    MGGCN_HIP(hipMemcpyAsync(&flag, w.flag, sizeof(int32_t), hipMemcpyDeviceToHost, s));
    MGGCN_HIP(hipStreamSynchronize(s));
    MGGCN_REQUIRE(flag == 0, MGGCN_E_BAD_CSR,
                  "malformed input pattern:%s%s%s", (flag & 1) ? " rowptr not monotone;" : "",
                  (flag & 2) ? " column index out of range;" : "",
                  (flag & 4) ? " row not strictly ascending;" : "");
  }

  if (n_rows > 0) {
    count_rows<IT><<<(unsigned)ceil_div(n_rows, kThreads), kThreads, 0, s>>>(n_rows, n_cols, rowptr_in,
                                                                             colidx_in, w.counts);
    MGGCN_LAUNCH_CHECK();
  }
  if constexpr (sizeof(IT) == 4)
    rc = exclusive_scan_i32(w.counts, n_rows, rowptr_out, w.scan_tmp, s);
  else
    rc = exclusive_scan_i64(w.counts, n_rows, rowptr_out, reinterpret_cast<int64_t*>(w.scan_tmp), s);
  if (rc) return rc;
  IT total = 0;
  MGGCN_HIP(hipMemcpyAsync(&total, rowptr_out + n_rows, sizeof(IT), hipMemcpyDeviceToHost, s));
  MGGCN_HIP(hipStreamSynchronize(s));
  *nnz_out = total;
  return MGGCN_OK;
}

template <typename IT>
int normalize_impl(int32_t n_rows, int32_t n_cols, const IT* rowptr_in, const int32_t* colidx_in, int mode,
                   const int32_t* deg_row, const int32_t* deg_col, const IT* rowptr_out, int32_t* colidx_out,
                   float* val_out, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_common(n_rows, n_cols, rowptr_in, colidx_in, ws, ws_bytes);
  if (rc) return rc;
  MGGCN_REQUIRE(mode == MGGCN_NORM_SYM_SELFLOOP || mode == MGGCN_NORM_MEAN_IN, MGGCN_E_INVALID_ARG,
                "unknown normalisation mode %d", mode);
  MGGCN_REQUIRE(rowptr_out != nullptr, MGGCN_E_INVALID_ARG, "rowptr_out is NULL");
  if (n_rows == 0 || n_cols == 0) return MGGCN_OK;  // no entries: nothing to fill (outputs may be NULL)
  MGGCN_REQUIRE(colidx_out && val_out, MGGCN_E_INVALID_ARG, "colidx_out / val_out is NULL");
  MGGCN_REQUIRE(!(mode == MGGCN_NORM_SYM_SELFLOOP && n_rows != n_cols && (!deg_row || !deg_col)),
                MGGCN_E_INVALID_ARG,
                "symmetric normalisation of a rectangular %d x %d block needs deg_row and deg_col",
                n_rows, n_cols);
  if (n_rows == 0) return MGGCN_OK;
  hipStream_t s = as_stream(stream);
  NormWs w;
  carve(n_rows, n_cols, ws, &w);
  const unsigned row_blocks = (unsigned)ceil_div((int64_t)n_rows * 64, kThreads);
  if (mode == MGGCN_NORM_SYM_SELFLOOP) {
    fill_rows<true, IT><<<row_blocks, kThreads, 0, s>>>(n_rows, n_cols, rowptr_in, colidx_in, deg_row,
                                                    deg_col, rowptr_out, colidx_out, val_out);
    MGGCN_LAUNCH_CHECK();
    return MGGCN_OK;
  }
  fill_rows<false, IT><<<row_blocks, kThreads, 0, s>>>(n_rows, n_cols, rowptr_in, colidx_in, nullptr,
                                                   nullptr, rowptr_out, colidx_out, val_out);
  MGGCN_LAUNCH_CHECK();
  IT nnz = 0;
  MGGCN_HIP(hipMemcpyAsync(&nnz, rowptr_out + n_rows, sizeof(IT), hipMemcpyDeviceToHost, s));
  MGGCN_HIP(hipStreamSynchronize(s));
  const int32_t* cc = deg_col;
  if (!cc) {
    zero_i32<<<(unsigned)ceil_div((int64_t)n_cols + 1, kThreads), kThreads, 0, s>>>(w.colcount,
                                                                                   (int64_t)n_cols + 1);
    MGGCN_LAUNCH_CHECK();
    if (nnz > 0) {
      column_histogram<<<(unsigned)ceil_div((int64_t)nnz, kThreads), kThreads, 0, s>>>((int64_t)nnz, colidx_out, w.colcount);
      MGGCN_LAUNCH_CHECK();
    }
    cc = w.colcount;
  }
  if (nnz > 0) {
    mean_values<<<(unsigned)ceil_div((int64_t)nnz, kThreads), kThreads, 0, s>>>((int64_t)nnz, colidx_out, cc, val_out);
    MGGCN_LAUNCH_CHECK();
  }
  return MGGCN_OK;
}

}  // namespace
}  // namespace mggcn

using namespace mggcn;

extern "C" {

size_t mggcn_csr_normalize_workspace_bytes(int32_t n_rows, int32_t n_cols) {
  if (n_rows < 0 || n_cols < 0) return 0;
  return carve(n_rows, n_cols, nullptr, nullptr);
}

int mggcn_csr_normalize_count(int32_t n_rows, int32_t n_cols, const int32_t* rowptr_in,
                              const int32_t* colidx_in, int validate, int32_t* rowptr_out,
                              int64_t* nnz_out, void* ws, size_t ws_bytes, void* stream) {
  return normalize_count_impl<int32_t>(n_rows, n_cols, rowptr_in, colidx_in, validate, rowptr_out, nnz_out, ws,
                                       ws_bytes, stream);
}

int mggcn_csr_normalize_count64(int32_t n_rows, int32_t n_cols, const int64_t* rowptr_in,
                                const int32_t* colidx_in, int validate, int64_t* rowptr_out,
                                int64_t* nnz_out, void* ws, size_t ws_bytes, void* stream) {
  return normalize_count_impl<int64_t>(n_rows, n_cols, rowptr_in, colidx_in, validate, rowptr_out, nnz_out, ws,
                                       ws_bytes, stream);
}

int mggcn_csr_normalize(int32_t n_rows, int32_t n_cols, const int32_t* rowptr_in,
                        const int32_t* colidx_in, int mode, const int32_t* deg_row,
                        const int32_t* deg_col, const int32_t* rowptr_out, int32_t* colidx_out,
                        float* val_out, void* ws, size_t ws_bytes, void* stream) {
  return normalize_impl<int32_t>(n_rows, n_cols, rowptr_in, colidx_in, mode, deg_row, deg_col, rowptr_out,
                                 colidx_out, val_out, ws, ws_bytes, stream);
}

int mggcn_csr_normalize64(int32_t n_rows, int32_t n_cols, const int64_t* rowptr_in,
                          const int32_t* colidx_in, int mode, const int32_t* deg_row,
                          const int32_t* deg_col, const int64_t* rowptr_out, int32_t* colidx_out,
                          float* val_out, void* ws, size_t ws_bytes, void* stream) {
  return normalize_impl<int64_t>(n_rows, n_cols, rowptr_in, colidx_in, mode, deg_row, deg_col, rowptr_out,
                                 colidx_out, val_out, ws, ws_bytes, stream);
}

}  // extern "C"
