// SpMM whose gathered operand is a bfloat16 copy of the dense matrix (fp32 accumulation, fp32
// output), and the conversion that makes the copy.  An extension beyond the paper, which keeps
// every operand in fp32: the gather of X rows is what the product spends its memory traffic on,
// and a 2-byte element halves it.  Same task tables, same kernel as the fp32 product.
#include "spmm_kernel.h"

#include <algorithm>

namespace mggcn {
namespace {

int launch_any_bf16(int vw, int lpr, const LaunchArgs& a) {
  switch (vw) {
    case 8: return launch_lpr<bf16_t, 8>(lpr, a);
    case 1: return launch_lpr<bf16_t, 1>(lpr, a);
    default: break;
  }
  return fail(MGGCN_E_UNSUPPORTED, "no bfloat16 SpMM kernel for vector width %d", vw);
}

// fp32 -> bfloat16, round to nearest, ties to even: add half a step minus one, plus the last
// kept bit, to the bit pattern and drop the low half.  Works unchanged for subnormals and carries
// into the exponent (up to infinity) where the value calls for it.  A NaN keeps its sign and
// upper payload and gets the quiet bit, so that dropping the low half cannot turn it into infinity.
__device__ inline uint32_t bf16_bits(float x) {
  const uint32_t u = __float_as_uint(x);
  if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) return (u >> 16) | 0x0040u;
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

__global__ __launch_bounds__(256) void f32_to_bf16_kernel(int64_t rows, int32_t cols, const float* __restrict__ src,
                                                           int64_t lds, uint16_t* __restrict__ dst, int64_t ldd,
                                                           int vec) {
  if (vec == 4) {  // 16-byte loads, 8-byte stores
    const int64_t per_row = cols / 4;
    const int64_t total = rows * per_row;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
      const int64_t r = i / per_row, q = i % per_row;
      const float4 t = *reinterpret_cast<const float4*>(src + r * lds + 4 * q);
      uint2 o;
      o.x = bf16_bits(t.x) | (bf16_bits(t.y) << 16);
      o.y = bf16_bits(t.z) | (bf16_bits(t.w) << 16);
      *reinterpret_cast<uint2*>(dst + r * ldd + 4 * q) = o;
    }
    return;
  }
  const int64_t total = rows * cols;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = i / cols, c = i % cols;
    dst[r * ldd + c] = (uint16_t)bf16_bits(src[r * lds + c]);
  }
}

}  // namespace
}  // namespace mggcn

using namespace mggcn;

extern "C" {

int mggcn_f32_to_bf16(int64_t rows, int32_t cols, const float* src, int64_t lds, uint16_t* dst, int64_t ldd,
                      void* stream) {
  MGGCN_REQUIRE(rows >= 0 && cols >= 0, MGGCN_E_INVALID_ARG, "negative size %lld x %d", (long long)rows, cols);
  MGGCN_REQUIRE(lds >= cols && ldd >= cols, MGGCN_E_INVALID_ARG, "leading dimension (lds %lld, ldd %lld) < cols %d",
                (long long)lds, (long long)ldd, cols);
  if (rows == 0 || cols == 0) return MGGCN_OK;
  MGGCN_REQUIRE(src != nullptr && dst != nullptr, MGGCN_E_INVALID_ARG, "src / dst is NULL");
  const bool v4 = cols % 4 == 0 && lds % 4 == 0 && ldd % 4 == 0 && aligned(src, 16) && aligned(dst, 8);
  const int64_t items = v4 ? rows * (cols / 4) : rows * (int64_t)cols;
  const int64_t blocks = std::min<int64_t>(ceil_div(items, 256), 256 * 32);
  f32_to_bf16_kernel<<<(unsigned)blocks, 256, 0, as_stream(stream)>>>(rows, cols, src, lds, dst, ldd, v4 ? 4 : 1);
  MGGCN_LAUNCH_CHECK();
  return MGGCN_OK;
}

int mggcn_spmm_bf16(const mggcn_graph* g, int op, const uint16_t* X, int64_t ldx, int32_t F, float beta,
                    int epilogue, float* Y, int64_t ldy, void* stream) {
  const int rc = spmm_check_args(g, op, X, ldx, (int)sizeof(uint16_t), F, beta, epilogue, Y, ldy);
  if (rc) return rc;
  const Orientation& o = (op == MGGCN_OP_N || g->symmetric) ? g->fwd : g->bwd;
  if (F == 0 || o.n_rows == 0) return MGGCN_OK;
  // eight elements per lane: one 16-byte gather load, two 16-byte stores of the fp32 result
  const int vw = (aligned(X, 16) && ldx % 8 == 0 && aligned(Y, 16) && ldy % 4 == 0) ? 8 : 1;
  return spmm_run(g, o, X, ldx, (int)sizeof(uint16_t), vw, F, beta, epilogue, Y, ldy, stream, launch_any_bf16);
}

}  // extern "C"
