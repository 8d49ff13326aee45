// Stand-alone probe: the inner loop of the fp32 GeMM rebuilt piece by piece on synthetic operand tiles, to
// see which piece costs matrix-pipe time and how much the operands' values matter.  Not part of the library.
//
// A workgroup of 4 wavefronts repeats `iters` k-steps of 32: matrix instructions (v_mfma_f32_32x32x2_f32) fed by
// LDS fragment reads from one of two stages; optionally the global loads of the next step (16-byte per lane, base
// in scalar registers) issued before the arithmetic; optionally their 16-byte stores into the other stage; one
// barrier per step; optionally the accumulators written out every 8 steps (a C tile of a product with K = 256).
//   narrow: 128 x 64 tile, 32 x 64 per wavefront (2 accumulators), 24 KiB loaded per step
//   wide:   128 x 128 tile, 64 x 64 per wavefront (4 accumulators), 32 KiB loaded per step
// Every global index is masked into its buffer (sizes are powers of two), every LDS index is bounded by the
// array shapes below.  Prints TFLOP/s per variant for constant, uniform random and zero operands.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

#define CHECK(x)                                                            \
  do {                                                                      \
    hipError_t e_ = (x);                                                    \
    if (e_ != hipSuccess) {                                                 \
      printf("%s failed: %s\n", #x, hipGetErrorString(e_));                 \
      exit(1);                                                              \
    }                                                                       \
  } while (0)

typedef float float16v __attribute__((ext_vector_type(16)));
typedef float vec4 __attribute__((ext_vector_type(4)));

// 16 bytes per lane from base (scalar registers) + offset (one vector register)
#define GLOAD(dst, voff, sbase) asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(dst) : "v"(voff), "s"(sbase) : "memory")

constexpr int kTileBytes = 16384;  // one operand tile of a step, as 256 lanes x 4 pieces of 16 bytes

__global__ void fill_random(float* p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    unsigned long long z = i * 0x9E3779B97F4A7C15ull + 0x1234567ull;
    z ^= z >> 31; z *= 0xBF58476D1CE4E5B9ull; z ^= z >> 29; z *= 0x94D049BB133111EBull; z ^= z >> 32;
    p[i] = (float)(unsigned)(z & 0xffffff) / 8388608.0f - 1.0f;  // uniform in [-1, 1)
  }
}

// FEED 0: LDS reads only; 1: + global loads, waited for and dropped; 2: + written to the other stage.
// WIDE: see above.  STORE: a C tile every 8 steps.
// g_mask: the buffer's size in bytes minus one, with the low 14 bits cleared (tile bases are multiples of 16 KiB
// and a tile's 16 KiB end inside the buffer); c_mask: number of floats of C minus one.
template <bool WIDE, int FEED, bool STORE>
__global__ __launch_bounds__(256) void loop(int iters, float* out, const char* __restrict__ G, size_t g_mask,
                                            float* __restrict__ C, size_t c_mask) {
  constexpr int BN = WIDE ? 128 : 64, TM = WIDE ? 2 : 1, TN = 2, WN = WIDE ? 2 : 1;
  constexpr int LDA = 128 + 4, LDB = BN + 4;
  constexpr int kStage = 32 * LDA + 32 * LDB;  // floats
  extern __shared__ __attribute__((aligned(16))) float lds[];  // [2][A: 32 x LDA | B: 32 x LDB]
  for (int i = threadIdx.x; i < 2 * kStage; i += 256) lds[i] = (float)(i % 7) * 0.125f;
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / WN, wn = wave % WN;  // wm < 4 / WN, so (wm * TM + TM) * 32 <= 128
  const int frow = lane >> 5, fcol = lane & 31;
  float16v acc[TM][TN];
  for (int i = 0; i < TM; ++i)
    for (int j = 0; j < TN; ++j)
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  const unsigned v = threadIdx.x * 16u;  // < 4096; + 12288 + 16 <= 16384
  constexpr int share = WIDE ? 1 : 2;     // log2 of the workgroups that read the same A tile (the N tiles of an M tile)
  for (int it = 0; it < iters; ++it) {
    const int cur = it & 1;
    vec4 h0, h1, h2, h3, h4, h5, h6, h7;
    if constexpr (FEED >= 1) {
      const size_t ta = (((size_t)(blockIdx.x >> share) * iters + it) * kTileBytes) & g_mask;
      const size_t tb = (((size_t)(blockIdx.x & ((1 << share) - 1)) * 64 + it) * kTileBytes) & 0xfc000 & g_mask;  // a 1 MiB region
      const char* pa = G + ta;
      const char* pb = G + tb;
      GLOAD(h0, v, pa); GLOAD(h1, v + 4096u, pa); GLOAD(h2, v + 8192u, pa); GLOAD(h3, v + 12288u, pa);
      GLOAD(h4, v, pb); GLOAD(h5, v + 4096u, pb);
      if constexpr (WIDE) { GLOAD(h6, v + 8192u, pb); GLOAD(h7, v + 12288u, pb); }
    }
    const float* As = lds + cur * kStage;
    const float* Bs = As + 32 * LDA;
    float a[16][TM], b[16][TN];
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
#pragma unroll
      for (int i = 0; i < TM; ++i) a[kk][i] = As[(2 * kk + frow) * LDA + (wm * TM + i) * 32 + fcol];
#pragma unroll
      for (int j = 0; j < TN; ++j) b[kk][j] = Bs[(2 * kk + frow) * LDB + (wn * TN + j) * 32 + fcol];
    }
#pragma unroll
    for (int kk = 0; kk < 16; ++kk)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[kk][i], b[kk][j], acc[i][j], 0, 0, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      __builtin_amdgcn_sched_group_barrier(0x008, TM * TN, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);
    }
    if constexpr (FEED >= 1) {
      if constexpr (WIDE) asm volatile("s_waitcnt vmcnt(0)" : "+v"(h0), "+v"(h1), "+v"(h2), "+v"(h3), "+v"(h4), "+v"(h5), "+v"(h6), "+v"(h7));
      else asm volatile("s_waitcnt vmcnt(0)" : "+v"(h0), "+v"(h1), "+v"(h2), "+v"(h3), "+v"(h4), "+v"(h5));
    }
    if constexpr (FEED == 2) {
      float* An = lds + (cur ^ 1) * kStage;
      float* Bn = An + 32 * LDA;
      const int row = threadIdx.x >> 5, c4 = 4 * (threadIdx.x & 31);  // rows 0..7 (+8, +16, +24), columns 0..127
      *reinterpret_cast<vec4*>(&An[(row + 0) * LDA + c4]) = h0; *reinterpret_cast<vec4*>(&An[(row + 8) * LDA + c4]) = h1;
      *reinterpret_cast<vec4*>(&An[(row + 16) * LDA + c4]) = h2; *reinterpret_cast<vec4*>(&An[(row + 24) * LDA + c4]) = h3;
      if constexpr (WIDE) {
        *reinterpret_cast<vec4*>(&Bn[(row + 0) * LDB + c4]) = h4; *reinterpret_cast<vec4*>(&Bn[(row + 8) * LDB + c4]) = h5;
        *reinterpret_cast<vec4*>(&Bn[(row + 16) * LDB + c4]) = h6; *reinterpret_cast<vec4*>(&Bn[(row + 24) * LDB + c4]) = h7;
      } else {
        const int rb = threadIdx.x >> 4, cb = 4 * (threadIdx.x & 15);  // rows 0..15 (+16), columns 0..63
        *reinterpret_cast<vec4*>(&Bn[(rb + 0) * LDB + cb]) = h4; *reinterpret_cast<vec4*>(&Bn[(rb + 16) * LDB + cb]) = h5;
      }
    }
    __syncthreads();
    if constexpr (STORE) {
      if ((it & 7) == 7) {  // rows of 256 floats, as C of an N = 256 product; every index is masked
        const size_t tile0 = ((size_t)(blockIdx.x >> share) * (iters / 8) + it / 8) * 128 * 256 +
                             (size_t)(blockIdx.x & ((1 << share) - 1)) * BN;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            const size_t corner = tile0 + (size_t)((wm * TM + i) * 32) * 256 + (wn * TN + j) * 32;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              C[(corner + (size_t)(8 * (r / 4) + 4 * frow + (r % 4)) * 256 + fcol) & c_mask] = acc[i][j][r];
              acc[i][j][r] = 0.f;
            }
          }
      }
    }
  }
  float s = 0.f;
  for (int i = 0; i < TM; ++i)
    for (int j = 0; j < TN; ++j)
      for (int r = 0; r < 16; ++r) s += acc[i][j][r];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;  // blocks <= 4096: out holds 4096 x 256 floats
}

struct Buffers {
  float* out;
  char* G;
  size_t g_bytes;
  float* C;
  size_t c_elems;
};

template <bool WIDE, int FEED, bool STORE>
void run(const char* name, const Buffers& b) {
  constexpr int BN = WIDE ? 128 : 64;
  constexpr size_t lds_bytes = (size_t)2 * (32 * (128 + 4) + 32 * (BN + 4)) * sizeof(float);
  static bool once = false;
  if (!once) {
    CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(loop<WIDE, FEED, STORE>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));
    once = true;
  }
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  const int blocks = WIDE ? 2048 : 3072, iters = 1000;  // four rounds of the workgroups resident at once
  const size_t g_mask = (b.g_bytes - 1) & ~(size_t)(kTileBytes - 1);
  float best = 1e30f;
  for (int rep = 0; rep < 3; ++rep) {
    CHECK(hipEventRecord(e0));
    loop<WIDE, FEED, STORE><<<blocks, 256, lds_bytes>>>(iters, b.out, b.G, g_mask, b.C, b.c_elems - 1);
    CHECK(hipGetLastError());
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    best = ms < best ? ms : best;
  }
  const double flop = (double)blocks * 4 * iters * (WIDE ? 64.0 : 32.0) * 4096.0;
  printf("  %-74s %7.1f TFLOP/s\n", name, flop / best / 1e9);
  fflush(stdout);
  CHECK(hipEventDestroy(e0));
  CHECK(hipEventDestroy(e1));
}

int main() {
  Buffers b;
  b.g_bytes = (size_t)1 << 32;  // 4 GiB of operand tiles
  b.c_elems = (size_t)1 << 29;  // 2 GiB of C
  CHECK(hipMalloc(&b.out, (size_t)4096 * 256 * sizeof(float)));
  CHECK(hipMalloc(&b.G, b.g_bytes));
  CHECK(hipMalloc(&b.C, b.c_elems * sizeof(float)));
  for (int pass = 0; pass < 3; ++pass) {
    if (pass == 0) { CHECK(hipMemset(b.G, 0x3c, b.g_bytes)); printf("operands: one constant (0x3c3c3c3c)\n"); }
    if (pass == 1) {
      fill_random<<<4096, 256>>>(reinterpret_cast<float*>(b.G), b.g_bytes / 4);
      CHECK(hipDeviceSynchronize());
      printf("operands: uniform random in [-1, 1)\n");
    }
    if (pass == 2) { CHECK(hipMemset(b.G, 0, b.g_bytes)); printf("operands: zero\n"); }
    if (pass == 0) {
      run<false, 0, false>("narrow: matrix instructions + LDS reads, two stages, one barrier per step", b);
      run<false, 1, false>("narrow: + global loads of the next step, dropped", b);
    }
    run<false, 2, false>("narrow (128 x 64, 32 x 64 per wavefront): the whole loop", b);
    run<false, 2, true>("narrow: the whole loop, C tile written every 8 steps", b);
    if (pass == 0) {
      run<true, 0, false>("wide: matrix instructions + LDS reads, two stages, one barrier per step", b);
      run<true, 1, false>("wide: + global loads of the next step, dropped", b);
    }
    run<true, 2, false>("wide (128 x 128, 64 x 64 per wavefront): the whole loop", b);
    run<true, 2, true>("wide: the whole loop, C tile written every 8 steps", b);
  }
  CHECK(hipFree(b.out));
  CHECK(hipFree(b.G));
  CHECK(hipFree(b.C));
  return 0;
}
