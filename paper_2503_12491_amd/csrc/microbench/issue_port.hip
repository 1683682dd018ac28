// Issue-rate microbenchmark for gfx950: how long the vector issue port of a SIMD is taken by
// v_fma_f32, v_exp_f32 and an MFMA, and how far an MFMA overlaps with vector work.  The score
// kernels spend their time on exactly this mix (logits on the matrix pipe; scaling, exponentials
// and sums on the vector pipe), so these figures give the bound their durations are compared to.
//
// Every test runs register-only loops in workgroups of 4 or 8 waves (wave i of a workgroup runs on
// SIMD i % 4), one or four workgroups per compute unit, so 1, 2, 4 or 8 waves share a SIMD; the
// figure printed is nanoseconds per instruction (or per MFMA with its K vector instructions) per
// SIMD.  Standalone program: prints a table, returns 0.
#include <hip/hip_runtime.h>

#include <cstdio>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

#define CHECK(x)                                                                   \
  do {                                                                             \
    hipError_t e = (x);                                                            \
    if (e != hipSuccess) {                                                         \
      printf("HIP error %s at line %d\n", hipGetErrorString(e), __LINE__);        \
      return 1;                                                                    \
    }                                                                              \
  } while (0)

enum Mode { kFma, kExp, kExpFma, kMfma32, kMfma16, kSplitWaves };

// kFma / kExp: 128 independent-enough instructions per iteration (8 chains).
// kExpFma: 32 groups per iteration of one v_exp_f32 followed by K v_fma_f32 on other registers.
// kMfma32 / kMfma16: 16 MFMAs per iteration (4 accumulator chains), each followed by K v_fma_f32.
// kSplitWaves: waves 4-7 of a workgroup run the 16 MFMAs, waves 0-3 run 16*K v_fma_f32, so every
// SIMD holds one wave of each kind per workgroup.
template <int MODE, int K>
__global__ __launch_bounds__(512) void issue_loop(float* out, int iters, float seed) {
  float v[8];
  for (int i = 0; i < 8; ++i) v[i] = seed + i + threadIdx.x * 1e-3f;
  f32x16 acc[4] = {};
  f32x4 small[4] = {};
  bf16x8 a, b;
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(seed * 0.01f);
    b[i] = (__bf16)(seed * 0.02f);
  }
  const bool mfma_wave = MODE != kSplitWaves || ((threadIdx.x >> 8) & 1);
  const bool fma_wave = MODE != kSplitWaves || !((threadIdx.x >> 8) & 1);
  for (int it = 0; it < iters; ++it) {
    if (MODE == kExpFma) {
#pragma unroll
      for (int r = 0; r < 32; ++r) {
        asm volatile("v_exp_f32 %0, %0" : "+v"(small[r & 3][r >> 3]));
#pragma unroll
        for (int i = 0; i < K; ++i) asm volatile("v_fma_f32 %0, %0, %1, %0" : "+v"(v[(r * K + i) & 7]) : "v"(seed));
      }
    } else if (MODE == kFma || MODE == kExp) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          if (MODE == kFma) asm volatile("v_fma_f32 %0, %0, %1, %0" : "+v"(v[i]) : "v"(seed));
          else asm volatile("v_exp_f32 %0, %0" : "+v"(v[i]));
        }
    } else {
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          if (mfma_wave) {
            if (MODE == kMfma16) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(small[c]) : "v"(a), "v"(b));
            else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[c]) : "v"(a), "v"(b));
          }
          if (fma_wave) {
#pragma unroll
            for (int i = 0; i < K; ++i) asm volatile("v_fma_f32 %0, %0, %1, %0" : "+v"(v[i & 7]) : "v"(seed));
          }
        }
    }
  }
  float s = 0;
  for (int i = 0; i < 8; ++i) s += v[i];
  for (int c = 0; c < 4; ++c) {
    for (int i = 0; i < 16; ++i) s += acc[c][i];
    for (int i = 0; i < 4; ++i) s += small[c][i];
  }
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <int MODE, int K>
int run(const char* name, int threads, double per_iter, const char* unit, float* out, int waves_per_unit = 1,
        int blocks_per_cu = 4) {
  const int iters = 2000 * 4 / blocks_per_cu, blocks = 256 * blocks_per_cu;
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  hipLaunchKernelGGL((issue_loop<MODE, K>), dim3(blocks), dim3(threads), 0, 0, out, 10, 1.0f);
  CHECK(hipDeviceSynchronize());
  CHECK(hipEventRecord(e0));
  hipLaunchKernelGGL((issue_loop<MODE, K>), dim3(blocks), dim3(threads), 0, 0, out, iters, 1.0f);
  CHECK(hipEventRecord(e1));
  CHECK(hipEventSynchronize(e1));
  float ms;
  CHECK(hipEventElapsedTime(&ms, e0, e1));
  // wave-iterations a SIMD works through; in the split test a unit is one iteration of each kind of wave
  const double simd_iters = (double)blocks * (threads / 64) / 1024.0 * iters / waves_per_unit;
  printf("%-44s %8.3f ms  %8.2f ns per %s\n", name, ms, ms * 1e6 / simd_iters / per_iter, unit);
  fflush(stdout);
  CHECK(hipEventDestroy(e0));
  CHECK(hipEventDestroy(e1));
  return 0;
}

int main() {
  float* out;
  CHECK(hipMalloc(&out, 256 * 4 * 512 * sizeof(float)));
  int rc = 0;
  rc |= run<kFma, 0>("v_fma_f32, 1 wave/SIMD", 256, 128, "instruction", out, 1, 1);
  rc |= run<kFma, 0>("v_fma_f32, 2 waves/SIMD", 512, 128, "instruction", out, 1, 1);
  rc |= run<kFma, 0>("v_fma_f32, 4 waves/SIMD", 256, 128, "instruction", out);
  rc |= run<kFma, 0>("v_fma_f32, 8 waves/SIMD", 512, 128, "instruction", out);
  rc |= run<kExp, 0>("v_exp_f32, 1 wave/SIMD", 256, 128, "instruction", out, 1, 1);
  rc |= run<kExp, 0>("v_exp_f32, 4 waves/SIMD", 256, 128, "instruction", out);
  rc |= run<kExpFma, 2>("v_exp_f32 + 2 v_fma_f32, 4 waves/SIMD", 256, 32, "group", out);
  rc |= run<kExpFma, 4>("v_exp_f32 + 4 v_fma_f32, 4 waves/SIMD", 256, 32, "group", out);
  rc |= run<kMfma32, 0>("mfma 32x32x16 bf16 alone, 1 wave/SIMD", 256, 16, "MFMA", out, 1, 1);
  rc |= run<kMfma32, 0>("mfma 32x32x16 bf16 alone, 4 waves/SIMD", 256, 16, "MFMA", out);
  rc |= run<kMfma32, 4>("mfma 32x32x16 bf16 + 4 fma each, 4 waves/SIMD", 256, 16, "MFMA", out);
  rc |= run<kMfma32, 6>("mfma 32x32x16 bf16 + 6 fma each, 4 waves/SIMD", 256, 16, "MFMA", out);
  rc |= run<kMfma32, 8>("mfma 32x32x16 bf16 + 8 fma each, 4 waves/SIMD", 256, 16, "MFMA", out);
  rc |= run<kMfma32, 12>("mfma 32x32x16 bf16 + 12 fma each, 4 waves/SIMD", 256, 16, "MFMA", out);
  rc |= run<kMfma32, 16>("mfma 32x32x16 bf16 + 16 fma each, 4 waves/SIMD", 256, 16, "MFMA", out);
  rc |= run<kMfma32, 8>("mfma 32x32x16 bf16 + 8 fma each, 1 wave/SIMD", 256, 16, "MFMA", out, 1, 1);
  rc |= run<kMfma32, 16>("mfma 32x32x16 bf16 + 16 fma each, 1 wave/SIMD", 256, 16, "MFMA", out, 1, 1);
  rc |= run<kMfma32, 8>("mfma 32x32x16 bf16 + 8 fma each, 2 waves/SIMD", 512, 16, "MFMA", out, 1, 1);
  rc |= run<kMfma32, 12>("mfma 32x32x16 bf16 + 12 fma each, 2 waves/SIMD", 512, 16, "MFMA", out, 1, 1);
  rc |= run<kMfma32, 16>("mfma 32x32x16 bf16 + 16 fma each, 2 waves/SIMD", 512, 16, "MFMA", out, 1, 1);
  rc |= run<kMfma32, 8>("mfma 32x32x16 bf16 + 8 fma each, 8 waves/SIMD", 512, 16, "MFMA", out);
  rc |= run<kMfma32, 16>("mfma 32x32x16 bf16 + 16 fma each, 8 waves/SIMD", 512, 16, "MFMA", out);
  rc |= run<kMfma16, 0>("mfma 16x16x32 bf16 alone, 4 waves/SIMD", 256, 16, "MFMA", out);
  rc |= run<kMfma16, 4>("mfma 16x16x32 bf16 + 4 fma each, 4 waves/SIMD", 256, 16, "MFMA", out);
  rc |= run<kMfma16, 8>("mfma 16x16x32 bf16 + 8 fma each, 4 waves/SIMD", 256, 16, "MFMA", out);
  rc |= run<kMfma16, 16>("mfma 16x16x32 bf16 + 16 fma each, 4 waves/SIMD", 256, 16, "MFMA", out);
  rc |= run<kSplitWaves, 8>("1+1 waves/SIMD: 16 mfma 32x32x16 | 128 fma", 512, 16, "MFMA (+8 fma in the other wave)", out, 2, 1);
  rc |= run<kSplitWaves, 16>("1+1 waves/SIMD: 16 mfma 32x32x16 | 256 fma", 512, 16, "MFMA (+16 fma in the other wave)", out, 2, 1);
  rc |= run<kSplitWaves, 8>("4+4 waves/SIMD: 16 mfma 32x32x16 | 128 fma", 512, 16, "MFMA (+8 fma in the other wave)", out, 2);
  rc |= run<kSplitWaves, 16>("4+4 waves/SIMD: 16 mfma 32x32x16 | 256 fma", 512, 16, "MFMA (+16 fma in the other wave)", out, 2);
  CHECK(hipFree(out));
  return rc;
}
