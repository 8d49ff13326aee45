// Device helpers shared by the SpMM kernels: vector loads along the feature dimension and the
// fused epilogue / masked store of an output row.
#pragma once

#include <hip/hip_runtime.h>

#include "../../include/mggcn.h"

namespace mggcn {

template <int VW>
__device__ inline void load_row(const float* __restrict__ p, int nf, float (&x)[VW]) {
  if (nf == VW) {
    if constexpr (VW % 4 == 0) {
#pragma unroll
      for (int q = 0; q < VW / 4; ++q) {
        const float4 t = reinterpret_cast<const float4*>(p)[q];
        x[4 * q] = t.x; x[4 * q + 1] = t.y; x[4 * q + 2] = t.z; x[4 * q + 3] = t.w;
      }
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

// streaming: nothing reads these values again before they leave the caches (the last write of a row
// of Y), so the stores are marked non-temporal and do not displace gathered rows of X: the
// transposed product of the 13.9 M x 111 M row block, a third of whose traffic is the write of its
// 111 M output rows, went from 33.5 to 31.7 ms.  Rows that a later column panel adds to keep the
// plain stores (all of them streamed, the 16-panel products of the medium graph were 1.4 % slower).
template <int VW>
__device__ inline void store_out(float* __restrict__ dst, int nf, const float (&a)[VW], float beta,
                                 int epi, bool final_row, bool streaming = false) {
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
    if constexpr (VW % 4 == 0) {
      typedef float float4v __attribute__((ext_vector_type(4)));
      float4v* out = reinterpret_cast<float4v*>(dst);
      if (streaming) {
        // The address passes through an empty asm statement so that the optimiser cannot fold the two
        // branches into one plain store (it would, dropping the non-temporal mark); it is typed as a
        // global-memory address so that the store stays a global one.
        typedef __attribute__((address_space(1))) float4v* global_float4v_ptr;
        global_float4v_ptr gout = (global_float4v_ptr)out;
        asm volatile("" : "+v"(gout));
#pragma unroll
        for (int q = 0; q < VW / 4; ++q) {
          const float4v t = {r[4 * q], r[4 * q + 1], r[4 * q + 2], r[4 * q + 3]};
          __builtin_nontemporal_store(t, gout + q);
        }
      } else {
#pragma unroll
        for (int q = 0; q < VW / 4; ++q) {
          const float4v t = {r[4 * q], r[4 * q + 1], r[4 * q + 2], r[4 * q + 3]};
          out[q] = t;
        }
      }
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

// Whole-vector load of VW floats.  The tail lane of a row may read up to VW-1 floats past F:
// they lie inside the row's leading dimension (ld is a multiple of VW on this path) and only
// feed accumulator components that are never stored.
template <int VW>
__device__ inline void load_vec(const float* __restrict__ p, float (&x)[VW]) {
  static_assert(VW == 4 || VW == 2 || VW == 1, "fp32 gathers are 16, 8 or 4 bytes per lane");
  if constexpr (VW == 4) {
    const float4 t = *reinterpret_cast<const float4*>(p);
    x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
  } else if constexpr (VW == 2) {
    const float2 t = *reinterpret_cast<const float2*>(p);
    x[0] = t.x; x[1] = t.y;
  } else {
    x[0] = p[0];
  }
}

}  // namespace mggcn
