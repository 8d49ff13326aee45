// Internal helpers of the mggcn HIP library: error reporting, argument checks, small
// device utilities.  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <exception>
#include <new>

#include "../../include/mggcn.h"

namespace mggcn {

// thread-local message behind mggcn_last_error()
char* error_buffer();
int fail(int code, const char* fmt, ...);

#define MGGCN_REQUIRE(cond, code, ...)                 \
  do {                                                 \
    if (!(cond)) return ::mggcn::fail((code), __VA_ARGS__); \
  } while (0)

#define MGGCN_HIP(expr)                                                                   \
  do {                                                                                    \
    hipError_t e_ = (expr);                                                               \
    if (e_ != hipSuccess)                                                                 \
      return ::mggcn::fail(MGGCN_E_HIP, "%s failed: %s", #expr, hipGetErrorString(e_));   \
  } while (0)

#define MGGCN_LAUNCH_CHECK()                                                                  \
  do {                                                                                        \
    hipError_t e_ = hipGetLastError();                                                        \
    if (e_ != hipSuccess)                                                                     \
      return ::mggcn::fail(MGGCN_E_HIP, "kernel launch failed at %s:%d: %s", __FILE__, __LINE__, \
                           hipGetErrorString(e_));                                            \
  } while (0)

// Body of an entry point that builds host-side tables: a C caller never sees a C++ exception.
template <class Fn>
int guarded(Fn&& body) {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    return fail(MGGCN_E_NO_MEMORY, "out of host memory");
  } catch (const std::exception& e) {
    return fail(MGGCN_E_NO_MEMORY, "host-side failure: %s", e.what());
  }
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

constexpr size_t kWsAlign = 256;

// Bump allocator over a caller-provided workspace.
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* p) : base(static_cast<char*>(p)) {}
  template <class T>
  T* take(size_t count) {
    T* r = reinterpret_cast<T*>(base + off);
    off += align_up(count * sizeof(T), kWsAlign);
    return r;
  }
};

inline hipStream_t as_stream(void* s) { return static_cast<hipStream_t>(s); }

// Exclusive prefix sum of `n` int32 counts (device), result in out[0..n] (n+1 entries,
// out[n] = total).  tmp needs scan_tmp_ints(n) int32 entries.  Three plain passes, no
// inter-block waiting.
size_t scan_tmp_ints(int64_t n);
int exclusive_scan_i32(const int32_t* counts, int64_t n, int32_t* out, int32_t* tmp, hipStream_t s);
// The same with 64-bit offsets (totals beyond 2^31); tmp needs scan_tmp_ints(n) int64 entries.
int exclusive_scan_i64(const int32_t* counts, int64_t n, int64_t* out, int64_t* tmp, hipStream_t s);

// Stable radix sort of n (key, value) pairs of 32 unsigned bits by the low key_bits bits of the key
// (sort.hip).  vals_in == nullptr sorts the positions 0..n-1 (an argsort).  keys_in / vals_in are not
// written; tmp needs radix_sort_tmp_bytes(n) bytes, 256-byte aligned.  n < 2^32.
size_t radix_sort_tmp_bytes(int64_t n);
int radix_sort_pairs(const uint32_t* keys_in, const uint32_t* vals_in, uint32_t* keys_out, uint32_t* vals_out,
                     int64_t n, int key_bits, void* tmp, hipStream_t s);

// The GeMM behind mggcn_gemm (pieces = false) and mggcn_gemm_bf16x3 (pieces = true).
int gemm_run(bool pieces, int opA, int opB, int64_t M, int64_t N, int64_t K, const float* A, int64_t lda,
             const float* B, int64_t ldb, float beta, int epilogue, float* C, int64_t ldc, void* ws,
             size_t ws_bytes, void* stream);

}  // namespace mggcn
