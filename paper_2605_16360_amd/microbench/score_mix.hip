// Instruction-mix ceiling of scoring pass 1 (row log-sum-exp, paper Sec. 3) on gfx950, with no memory traffic at all.
//
// Per 32-key sub-tile and wave, pass 1 issues 8 v_mfma_f32_32x32x16_bf16 (two query sub-tiles, d = 64) and, on the
// 2 x 16 logits per lane that they produce, 32 x (v_fma_f32, v_exp_f32, v_add_f32).  This program runs exactly that
// mix out of registers, at the kernel's occupancy (256-thread workgroups, WPE waves per SIMD), in three forms:
//   mfma    the 8 MFMAs only
//   vector  the 96 vector instructions only
//   both    the MFMAs, then the vector work on their results (the kernel's shape)
// and prints, for each, the elapsed time and the fraction of the matrix pipe's peak it corresponds to
// (8 MFMAs x 32 cycles per sub-tile and wave against the elapsed cycles at 2.4 GHz).  If the two kinds of work ran
// side by side, "both" would take as long as the longer of the two; it takes nearly their sum, and that sum is the
// ceiling that the scoring kernel is measured against.
//
// Build and run (one MI355X):
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         -o paper_2605_16360_amd/microbench/score_mix paper_2605_16360_amd/microbench/score_mix.hip
//   ./paper_2605_16360_amd/microbench/score_mix
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define CHECK(x)                                                            \
  do {                                                                      \
    hipError_t e_ = (x);                                                    \
    if (e_ != hipSuccess) {                                                 \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
      exit(1);                                                              \
    }                                                                       \
  } while (0)

__device__ __forceinline__ f32x16 mm(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 zero16() { return f32x16{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}; }

enum Form { kMfma, kVector, kBoth };

// LDSKB keeps further workgroups off the CU, so that WPE is the occupancy that runs
template <int FORM, int WPE, int LDSKB>
__global__ __launch_bounds__(256, WPE) void mix_kernel(float* out, int iters, float seed) {
  __shared__ float pad[LDSKB * 256];
  pad[threadIdx.x] = seed;
  __syncthreads();
  const float sd = pad[threadIdx.x & 63];
  bf16x8 a[4], b[2][4];
  for (int kk = 0; kk < 4; ++kk)
    for (int i = 0; i < 8; ++i) {
      a[kk][i] = (__bf16)(sd * 0.01f * (i + kk));
      b[0][kk][i] = (__bf16)(sd * 0.02f * (i - kk));
      b[1][kk][i] = (__bf16)(sd * 0.03f * (i + 2 * kk));
    }
  const float c = 0.18f * sd, nref = -1.0f * sd;
  float l0 = 0, l1 = 0, l2 = 0, l3 = 0;
  auto vec16 = [&](const f32x16& acc) {
#pragma unroll
    for (int r = 0; r < 16; r += 4) {
      l0 += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[r + 0], c, nref));
      l1 += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[r + 1], c, nref));
      l2 += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[r + 2], c, nref));
      l3 += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[r + 3], c, nref));
    }
  };
  if constexpr (FORM == kMfma) {
    f32x16 acc[2] = {zero16(), zero16()};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int cs = 0; cs < 2; ++cs)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) acc[cs] = mm(a[kk], b[cs][kk], acc[cs]);
    }
    l0 = acc[0][0] + acc[1][1];
  } else if constexpr (FORM == kVector) {
    f32x16 acc[2];
    for (int i = 0; i < 16; ++i) {
      acc[0][i] = sd * i;
      acc[1][i] = sd * (i + 16);
    }
    for (int it = 0; it < iters; ++it) {
      vec16(acc[0]);
      vec16(acc[1]);
      acc[0][it & 15] += l0 * 1e-30f;  // keeps the iterations distinct
    }
  } else {
    for (int it = 0; it < iters; ++it) {
      f32x16 acc[2];
#pragma unroll
      for (int cs = 0; cs < 2; ++cs) {
        acc[cs] = zero16();
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) acc[cs] = mm(a[kk], b[cs][kk], acc[cs]);
      }
      vec16(acc[0]);
      vec16(acc[1]);
      a[0][0] += (__bf16)l0;  // keeps the iterations distinct
    }
  }
  out[blockIdx.x * 256 + threadIdx.x] = (l0 + l1) + (l2 + l3);
}

template <int FORM, int WPE, int LDSKB>
double run(const char* name, float* out, int iters) {
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  const int blocks = 256 * WPE;  // one per CU and occupancy slot
  mix_kernel<FORM, WPE, LDSKB><<<blocks, 256>>>(out, 10, 1.0f);
  CHECK(hipGetLastError());
  CHECK(hipDeviceSynchronize());
  CHECK(hipEventRecord(e0));
  mix_kernel<FORM, WPE, LDSKB><<<blocks, 256>>>(out, iters, 1.0f);
  CHECK(hipGetLastError());
  CHECK(hipEventRecord(e1));
  CHECK(hipEventSynchronize(e1));
  float ms;
  CHECK(hipEventElapsedTime(&ms, e0, e1));
  const double mfma_cycles = (double)WPE * iters * 8 * 32;  // matrix-pipe cycles per SIMD
  if (FORM == kVector) printf("%-8s %d waves/SIMD  %8.3f ms\n", name, WPE, ms);
  else printf("%-8s %d waves/SIMD  %8.3f ms   fraction of the MFMA peak at 2.4 GHz: %.3f\n", name, WPE, ms, mfma_cycles / (ms * 1e-3 * 2.4e9));
  fflush(stdout);
  CHECK(hipEventDestroy(e0));
  CHECK(hipEventDestroy(e1));
  return ms;
}

int main() {
  float* out;
  CHECK(hipMalloc(&out, (size_t)256 * 4 * 256 * sizeof(float)));
  const int iters = 40000;
  const double m3 = run<kMfma, 3, 40>("mfma", out, iters);
  const double v3 = run<kVector, 3, 40>("vector", out, iters);
  const double b3 = run<kBoth, 3, 40>("both", out, iters);
  printf("3 waves/SIMD: both / (mfma + vector) = %.3f, both / max(mfma, vector) = %.3f\n", b3 / (m3 + v3), b3 / (m3 > v3 ? m3 : v3));
  const double m4 = run<kMfma, 4, 30>("mfma", out, iters);
  const double v4 = run<kVector, 4, 30>("vector", out, iters);
  const double b4 = run<kBoth, 4, 30>("both", out, iters);
  printf("4 waves/SIMD: both / (mfma + vector) = %.3f, both / max(mfma, vector) = %.3f\n", b4 / (m4 + v4), b4 / (m4 > v4 ? m4 : v4));
  CHECK(hipFree(out));
  return 0;
}
