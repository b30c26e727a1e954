// What the matrix pipe of this part sustains, apart from any kernel design: a register-only loop
// of v_mfma_f32_32x32x16_bf16 on all 256 CUs (8 waves per CU, two per SIMD, independent
// accumulators, no memory traffic), once with the same operand registers for every MFMA and once
// cycling through eight different pseudo-random operand pairs (the power drawn depends on how many
// operand bits toggle between issues, and the clock follows the power limit); and whether the
// vector ALU work of one wave (fma + exp2 + add, the softmax's inner operations) runs in the shadow
// of another wave's, or its own, MFMAs.  Prints PFLOP/s and the clock implied by 32 cycles per MFMA.
// Measurement aid only: nothing in the library uses it.
//   hipcc --offload-arch=gfx950 -O3 mfma_sustained.hip -o mfma_sustained && ./mfma_sustained
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));

#define CK(x)                                                                   \
  do {                                                                          \
    hipError_t e_ = (x);                                                        \
    if (e_ != hipSuccess) {                                                     \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);     \
      exit(1);                                                                  \
    }                                                                           \
  } while (0)

__device__ inline unsigned mix(unsigned x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}

// MODE 0: MFMA, constant operands   1: MFMA, eight random operand pairs in turn
//      2: vector work only          3: waves 0-3 MFMA, waves 4-7 vector work (same SIMDs)
//      4: every wave alternates one MFMA and one group of vector work
template <int MODE>
__global__ void __launch_bounds__(512) kern(float* out, int iters) {
  const int wave = threadIdx.x >> 6;
  floatx16_t acc[4];
  for (int i = 0; i < 4; ++i)
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  bf16x8_t a[8], b[8];
  for (int p = 0; p < 8; ++p)
    for (int i = 0; i < 8; ++i) {
      const unsigned h = mix((blockIdx.x * 512 + threadIdx.x) * 64 + p * 8 + i);
      const int q = MODE == 1 ? p : 0;                       // MODE 0: one pair for all
      const unsigned hq = mix((blockIdx.x * 512 + threadIdx.x) * 64 + q * 8 + i);
      a[p][i] = (__bf16)(((MODE == 1 ? h : hq) & 0xffff) / 32768.0f - 1.0f);
      b[p][i] = (__bf16)((((MODE == 1 ? h : hq) >> 16) & 0xffff) / 32768.0f * 0.02f - 0.02f);
    }
  float v[32];
  for (int i = 0; i < 32; ++i) v[i] = 0.01f * (threadIdx.x + i);
  float sum = 0.f;
  const bool do_mfma = MODE <= 1 || (MODE == 3 && wave < 4);
  const bool do_valu = MODE == 2 || (MODE == 3 && wave >= 4);
  for (int it = 0; it < iters; ++it) {
    if (MODE == 4) {
#pragma unroll
      for (int j = 0; j < 32; ++j) {
        acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[0], acc[j & 3], 0, 0, 0);
        const float p = __builtin_amdgcn_exp2f(fmaf(v[j], 0.125f, -1.0f));
        sum += p; v[j] = p;
      }
    } else {
      if (do_mfma) {
#pragma unroll
        for (int j = 0; j < 32; ++j)
          acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j & 7], b[j & 7], acc[j & 3], 0, 0, 0);
      }
      if (do_valu) {
#pragma unroll
        for (int j = 0; j < 32; ++j) {
          const float p = __builtin_amdgcn_exp2f(fmaf(v[j], 0.125f, -1.0f));
          sum += p; v[j] = p;
        }
      }
    }
  }
  float r = sum;
  for (int i = 0; i < 4; ++i)
    for (int k = 0; k < 16; ++k) r += acc[i][k];
  out[blockIdx.x * 512 + threadIdx.x] = r;
}

template <int MODE>
static void run(const char* name, float* out, int iters, double mfma_per_simd_iter) {
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  hipLaunchKernelGGL(kern<MODE>, dim3(256), dim3(512), 0, 0, out, 100);
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(e0));
  hipLaunchKernelGGL(kern<MODE>, dim3(256), dim3(512), 0, 0, out, iters);
  CK(hipEventRecord(e1));
  CK(hipDeviceSynchronize());
  float ms = 0.f;
  CK(hipEventElapsedTime(&ms, e0, e1));
  const double us_iter = ms * 1e3 / iters;
  printf("%-58s %8.3f us per iteration", name, us_iter);
  if (mfma_per_simd_iter > 0) {
    const double flops = mfma_per_simd_iter * 1024.0 * 32768.0 * iters;      // 1024 SIMDs, 32x32x16x2 per MFMA
    printf("   %6.3f PFLOP/s   clock >= %.2f GHz", flops / (ms * 1e-3) / 1e15, mfma_per_simd_iter * 32.0 / us_iter / 1e3);
  }
  printf("\n");
}

int main() {
  float* out;
  CK(hipMalloc(&out, 256 * 512 * sizeof(float)));
  const int iters = 40000;
  run<0>("MFMA only, same operand registers every time", out, iters, 64);
  run<1>("MFMA only, eight pseudo-random operand pairs in turn", out, iters, 64);
  run<2>("vector work only (32 x fma+exp2+add per wave and iteration)", out, iters, 0);
  run<3>("waves 0-3 MFMA, waves 4-7 vector work", out, iters, 32);
  run<4>("every wave alternates MFMA and vector work", out, iters, 64);
  CK(hipFree(out));
  return 0;
}
