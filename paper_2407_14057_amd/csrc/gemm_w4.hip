// bf16 GEMM, 256x256x64 tile on FOUR waves, one per SIMD, each holding a 128x128 block of the
// product (16 accumulator blocks of 32x32 = 256 registers, which the compiler keeps in the
// accumulation half of the 512-register file a lone wave of a SIMD has).  Against the 8-wave
// ping-pong form (two waves per SIMD, 64x128 each) a wave reads 8 operand fragments from LDS
// per 16 MFMAs instead of 6 per 8 -- a third less LDS traffic per FLOP -- and there is one
// workgroup barrier per K step instead of four.  There is no second wave to hide anything behind:
// the wave's own stream interleaves the LDS reads of the next K slice and the global -> LDS copies
// of the step after next with its MFMAs, one memory instruction per MFMA slot.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.h"
#include "gemm_shared.h"

namespace lz {

template <int EPI>
__global__ void __launch_bounds__(256)
gemm_w4_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ W,
               uint16_t* __restrict__ C, const uint16_t* __restrict__ R, int M, int N, int K, int lda,
               int ldw, int ldc, int tiles_m, int tiles_n, int group_m, EpiArgs ra) {
  constexpr int WM = 2, WN = 2, TM = 4, TN = 4, NWAVES = 4;
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  constexpr int A_INSTR = BM / 8 / NWAVES, W_INSTR = BN / 8 / NWAVES;    // 8 + 8 copies per wave and K step
  constexpr int NCOPY = A_INSTR + W_INSTR;
  constexpr int STAGE_BYTES = (BM + BN) * ROW_BYTES;
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  if ((int)blockIdx.x >= tiles_m * tiles_n) {     // side job (see EpiArgs): Eq. 1 scores
    const int sb = (int)blockIdx.x - tiles_m * tiles_n;
    score_finish_block<true>(ra.sf_z, ra.sf_stat, ra.sf_s, ra.sf_cu, ra.sf_n_single, ra.sf_heads,
                             ra.sf_z_ld, ra.sf_cu_z, true, sb / ra.sf_blocks_per_seq,
                             (sb % ra.sf_blocks_per_seq) * (int)blockDim.x, (float2*)lds);
    return;
  }
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / WN, wn = wave % WN;
  int tile_m, tile_n;
  workgroup_tile((int)blockIdx.x, tiles_m, tiles_n, group_m, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int crow = lane >> 3;
  uint32_t a_off[A_INSTR], w_off[W_INSTR];
#pragma unroll
  for (int q = 0; q < A_INSTR; ++q) {
    const int tr = (wave * A_INSTR + q) * 8 + crow;
    const int cchunk = (lane & 7) ^ swz64(tr);
    int r = m0 + tr;
    r = r < M ? r : M - 1;
    if (ra.a_rows != nullptr) r = ra.a_rows[r];
    a_off[q] = (uint32_t)(((size_t)r * lda + cchunk * 8) * 2);
  }
#pragma unroll
  for (int q = 0; q < W_INSTR; ++q) {
    const int tr = (wave * W_INSTR + q) * 8 + crow;
    const int cchunk = (lane & 7) ^ swz64(tr);
    int r = n0 + tr;
    r = r < N ? r : N - 1;
    w_off[q] = (uint32_t)(((size_t)r * ldw + cchunk * 8) * 2);
  }
  const uint32_t wstep32 = (uint32_t)ra.w_step_bytes;
  // one of the wave's copies of a K step (uniform base + 32-bit lane offset; the launcher checks
  // that both operands span less than 4 GB)
  auto issue_one = [&](int stage, int kt, int q) {
    if (q < A_INSTR)
      g2l16((const char*)A + (uint32_t)(a_off[q] + (uint32_t)kt * (uint32_t)(BK * 2)),
            lds + stage * STAGE_BYTES + (wave * A_INSTR + q) * 1024);
    else
      g2l16((const char*)W + (uint32_t)(w_off[q - A_INSTR] + (uint32_t)kt * wstep32),
            lds + stage * STAGE_BYTES + BM * ROW_BYTES + (wave * W_INSTR + q - A_INSTR) * 1024);
  };

  uint32_t koff[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
    koff[ks] = (uint32_t)(((ks * 2 + (lane >> 5)) ^ swz64(lane & 31)) * 16);
  const uint32_t a_row = (uint32_t)((wm * TM * 32 + (lane & 31)) * ROW_BYTES);
  const uint32_t w_row = (uint32_t)(BM * ROW_BYTES + (wn * TN * 32 + (lane & 31)) * ROW_BYTES);

  floatx16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  bf16x8_t af[2][TM], wf[2][TN];

#define LZ_LOAD_FRAGS(buf, st, ks)                                                            \
  do {                                                                                        \
    _Pragma("unroll") for (int i = 0; i < TM; ++i)                                            \
        af[buf][i] = *(const bf16x8_t*)((st) + a_row + i * 32 * ROW_BYTES + koff[ks]);        \
    _Pragma("unroll") for (int j = 0; j < TN; ++j)                                            \
        wf[buf][j] = *(const bf16x8_t*)((st) + w_row + j * 32 * ROW_BYTES + koff[ks]);        \
  } while (0)
#define LZ_MFMAS(buf)                                                                         \
  do {                                                                                        \
    _Pragma("unroll") for (int i = 0; i < TM; ++i)                                            \
      _Pragma("unroll") for (int j = 0; j < TN; ++j)                                          \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[buf][j], af[buf][i],           \
                                                            acc[i][j], 0, 0, 0);              \
  } while (0)
  // a K slice: 16 MFMAs with the 8 fragment reads of the next slice behind the first 8
#define LZ_SCHED_READS()                                                                      \
  do {                                                                                        \
    _Pragma("unroll") for (int n = 0; n < TM + TN; ++n) {                                     \
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                      \
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                      \
    }                                                                                         \
    __builtin_amdgcn_sched_group_barrier(0x008, TM * TN - (TM + TN), 0);                      \
  } while (0)

  const int KT = K / BK;
#pragma unroll
  for (int q = 0; q < NCOPY; ++q) issue_one(0, 0, q);
  if (KT > 1) {
#pragma unroll
    for (int q = 0; q < NCOPY; ++q) issue_one(1, 1, q);
  }
  float rs[TM];
  load_row_scales<TM>(rs, ra, M, m0, wm, lane);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  LZ_LOAD_FRAGS(0, lds, 0);
  for (int kt = 0; kt < KT; ++kt) {
    const char* cur = lds + (kt & 1) * STAGE_BYTES;
    const char* nxt = lds + ((kt + 1) & 1) * STAGE_BYTES;
    __builtin_amdgcn_s_setprio(1);
    LZ_LOAD_FRAGS(1, cur, 1);
    LZ_MFMAS(0);
    LZ_SCHED_READS();
    LZ_LOAD_FRAGS(0, cur, 2);
    LZ_MFMAS(1);
    LZ_SCHED_READS();
    LZ_LOAD_FRAGS(1, cur, 3);
    LZ_MFMAS(0);
    LZ_SCHED_READS();
    __builtin_amdgcn_s_setprio(0);
    // every wave has its last fragments of this stage in registers, and step kt + 1 (copied during
    // the last slice of step kt - 1) has landed: the stage is free for step kt + 2
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    // last slice: its 16 MFMAs carry the step-after-next's 16 copies and the next step's first
    // 8 fragment reads, one copy behind every MFMA and a read behind every other
    const int kt_copy = kt + 2 < KT ? kt + 2 : KT - 1;     // (past the end: a harmless re-copy, no branch)
    if (kt + 1 < KT) LZ_LOAD_FRAGS(0, nxt, 0);
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[1][j], af[1][i], acc[i][j], 0, 0, 0);
        issue_one(kt & 1, kt_copy, i * TN + j);
      }
#pragma unroll
    for (int n = 0; n < NCOPY; ++n) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
      if ((n & 1) == 0) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_s_setprio(0);
  }
#undef LZ_LOAD_FRAGS
#undef LZ_MFMAS
#undef LZ_SCHED_READS
  // (the re-copies of the last two iterations are still in flight: nothing reads them, but the
  // staged output below reuses the stages, so they are drained first)
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  if (EPI == EPI_SWIGLU || !ra.stage_out) {
    gemm_epilogue<TM, TN, EPI>(acc, C, R, M, ldc, m0, n0, wm, wn, lane, ra, rs);
    return;
  }
  staged_tile_out<TM, TN, EPI, BM, BN, NWAVES>(acc, C, R, M, ldc, m0, n0, wm, wn, wave, lane, ra, rs, lds);
}

hipError_t launch_gemm_w4(const void* A, const void* W, void* C, const void* R, int M, int N, int K,
                          int lda, int ldw, int ldc, int epi, int group_m, const EpiArgs& ra,
                          hipStream_t st) {
  constexpr int BM = 256, BN = 256;
  constexpr int LDS_BYTES = 2 * (BM + BN) * ROW_BYTES;
  if (N % BN != 0) return hipErrorInvalidValue;
  if ((unsigned long long)M * lda * 2 >= (1ull << 32) ||
      (unsigned long long)N * (ra.w_blocked ? K : ldw) * 2 >= (1ull << 32))
    return hipErrorInvalidValue;
  const int tiles_m = (M + BM - 1) / BM, tiles_n = N / BN;
  EpiArgs ea = ra;
  ea.w_step_bytes = ra.w_blocked ? (unsigned long long)N * ROW_BYTES : (unsigned long long)ROW_BYTES;
  if (ra.w_blocked) ldw = BK;
  ea.sf_blocks_per_seq = (ea.sf_max_rows + 255) / 256;
  ea.stage_out = (epi == EPI_QKV_ROPE) ? (ra.d_model % BN == 0 && (ra.kv_dim > 0 ? ra.kv_dim : ra.d_model) % BN == 0)
                 : (epi != EPI_SWIGLU && ldc % 8 == 0 && ((uintptr_t)C & 15) == 0);
  const int side = ea.sf_z != nullptr ? ea.sf_blocks_per_seq * ea.sf_batch : 0;
  dim3 grid(tiles_m * tiles_n + side), block(256);
#define LZ_GEMM(E)                                                                               \
  do {                                                                                           \
    auto kern = gemm_w4_kernel<E>;                                                               \
    static bool attr_set = false;                                                                \
    if (!attr_set) {                                                                             \
      hipError_t e = hipFuncSetAttribute((const void*)kern,                                      \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES); \
      if (e != hipSuccess) return e;                                                             \
      attr_set = true;                                                                           \
    }                                                                                            \
    hipLaunchKernelGGL(kern, grid, block, LDS_BYTES, st, (const uint16_t*)A, (const uint16_t*)W, \
                       (uint16_t*)C, (const uint16_t*)R, M, N, K, lda, ldw, ldc, tiles_m,        \
                       tiles_n, group_m, ea);                                                    \
  } while (0)
  if (epi == EPI_STORE) LZ_GEMM(EPI_STORE);
  else if (epi == EPI_RESIDUAL) LZ_GEMM(EPI_RESIDUAL);
  else if (epi == EPI_SWIGLU) LZ_GEMM(EPI_SWIGLU);
  else if (epi == EPI_QKV_ROPE) {
    if (ra.head_dim == 64) LZ_GEMM(EPI_QKV_ROPE64);
    else LZ_GEMM(EPI_QKV_ROPE128);
  }
  else return hipErrorInvalidValue;
#undef LZ_GEMM
  return hipGetLastError();
}

}  // namespace lz
