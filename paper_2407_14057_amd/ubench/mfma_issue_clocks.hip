// Cycles per v_mfma_f32_32x32x16_bf16 as a wave sees them (s_memtime, which ticks at the shader
// clock), for several dependency patterns between consecutive MFMAs -- eight independent
// accumulators, one accumulator, dependent pairs, two and four accumulators in turn -- with one
// wave per SIMD and with two, on one CU and on all 256.  Together with the event time of the
// launch this also gives the clock the chip holds under that load.  Measurement aid only:
// nothing in the library uses it.
//   hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops mfma_issue_clocks.hip -o mfma_issue_clocks && ./mfma_issue_clocks
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#define CK(x)                                                                   \
  do {                                                                          \
    hipError_t e_ = (x);                                                        \
    if (e_ != hipSuccess) {                                                     \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);     \
      exit(1);                                                                  \
    }                                                                           \
  } while (0)
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16_t;
#define MF(a, b, c) c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0)
template <int MODE>
__global__ void __launch_bounds__(512) k(unsigned long long* out, float* sink, int iters) {
  bf16x8_t a[4], b[4];
  for (int i = 0; i < 4; ++i)
    for (int e = 0; e < 8; ++e) { a[i][e] = (__bf16)(float)(threadIdx.x % 7 + i + e); b[i][e] = (__bf16)(float)(threadIdx.x % 5 + i - e); }
  floatx16_t c[8];
  for (int i = 0; i < 8; ++i) for (int e = 0; e < 16; ++e) c[i][e] = 0.f;
  __syncthreads();
  unsigned long long t0 = __builtin_readcyclecounter();
  for (int it = 0; it < iters; ++it) {
    if (MODE == 0) {            // 8 independent accumulators, round robin (2 rounds)
#pragma unroll
      for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int i = 0; i < 8; ++i) MF(a[i & 3], b[(i >> 1) & 3], c[i]);
    } else if (MODE == 1) {     // one accumulator, dependent chain
#pragma unroll
      for (int i = 0; i < 16; ++i) MF(a[i & 3], b[(i >> 1) & 3], c[0]);
    } else if (MODE == 2) {     // dependent pairs
#pragma unroll
      for (int i = 0; i < 8; ++i) { MF(a[i & 3], b[(i >> 1) & 3], c[i]); MF(a[(i + 1) & 3], b[(i >> 1) & 3], c[i]); }
    } else if (MODE == 3) {     // 2 accumulators alternating
#pragma unroll
      for (int i = 0; i < 16; ++i) MF(a[i & 3], b[(i >> 1) & 3], c[i & 1]);
    } else if (MODE == 4) {     // 4 accumulators
#pragma unroll
      for (int i = 0; i < 16; ++i) MF(a[i & 3], b[(i >> 1) & 3], c[i & 3]);
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  unsigned long long t1 = __builtin_readcyclecounter();
  float s = 0.f;
  for (int i = 0; i < 8; ++i) for (int e = 0; e < 16; ++e) s += c[i][e];
  sink[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if ((threadIdx.x & 63) == 0) out[blockIdx.x * 8 + (threadIdx.x >> 6)] = t1 - t0;
}
template <int MODE>
void run(const char* name, int blocks, int threads) {
  unsigned long long* out; float* sink;
  CK(hipMalloc(&out, blocks * 8 * 8)); CK(hipMalloc(&sink, blocks * threads * 4));
  const int iters = 2000;
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  k<MODE><<<blocks, threads>>>(out, sink, 100);
  CK(hipEventRecord(e0));
  k<MODE><<<blocks, threads>>>(out, sink, iters);
  CK(hipEventRecord(e1));
  CK(hipDeviceSynchronize());
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  unsigned long long h[8]; CK(hipMemcpy(h, out, 64, hipMemcpyDeviceToHost));
  const int per_simd = threads / 256;                       // waves that share a SIMD
  const double ticks = (double)h[0] / (iters * 16.0);       // wave 0: cycles between two of ITS MFMAs
  const double ns = ms * 1e6 / (iters * 16.0 * per_simd);   // time per MFMA that a SIMD issues
  printf("%-34s %3d CUs, %d wave(s) per SIMD: wave 0 sees %.2f cycles per MFMA; a SIMD issues one every %.2f ns",
         name, blocks, per_simd, ticks, ns);
  // with two waves per SIMD the older wave is served first and ends early: its cycle count says
  // nothing about the clock
  if (per_simd == 1) printf(" -> clock %.3f GHz", ticks / ns);
  printf(", %.0f TFLOP/s over the CUs used\n", blocks * 4 * 32768.0 / ns / 1e3);
  CK(hipFree(out)); CK(hipFree(sink));
}
int main() {
  for (int blocks : {1, 256}) {
    run<0>("8 independent accumulators", blocks, 256);
    run<1>("1 accumulator (dependent chain)", blocks, 256);
    run<2>("dependent pairs", blocks, 256);
    run<3>("2 accumulators alternating", blocks, 256);
    run<4>("4 accumulators round robin", blocks, 256);
    run<0>("8 independent, 2 waves per SIMD", blocks, 512);
    run<2>("dependent pairs, 2 waves per SIMD", blocks, 512);
  }
  return 0;
}
