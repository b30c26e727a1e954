// 8-bit floating point variant of the projections' GEMM (an extension: the paper computes in
// 16-bit floating point).  Operands are OFP8 E4M3 codes with one fp32 scale per row (a token of
// the activations, an output feature of the weights), both K-contiguous:
//   C[m, n] = sa[m] * sw[n] * sum_k a[m, k] * w[n, k],   fp32 accumulation on the matrix cores
// (v_mfma_f32_32x32x64_f8f6f4: 64 K elements per instruction, twice the 16-bit rate), followed by
// the same epilogues as the 16-bit kernels.
//
// Two kernels: the row quantiser (16-bit floats -> codes + scale) and the tile kernel.
#include "common.h"
#include "gemm_shared.h"

namespace lz {

typedef int v4i_t __attribute__((ext_vector_type(4)));
typedef int v8i_t __attribute__((ext_vector_type(8)));

// ------------------------------------------------------------------------------------------
// Row quantiser: scale = max|row| / 448 (1 for an all-zero row), code = E4M3(x / scale), round
// to nearest even, magnitudes clamped to 448 before the conversion.  One workgroup per row; the
// row stays in registers between the maximum and the conversion (K <= 16384).
// ------------------------------------------------------------------------------------------
constexpr int Q8_CHUNKS = 8;                       // 16-byte chunks of the row per thread

__global__ void __launch_bounds__(256)
quantize_rows_f8_kernel(const uint16_t* __restrict__ x, int ldx, int K, uint8_t* __restrict__ q,
                        int ldq, float* __restrict__ scale) {
  __shared__ float red[4];
  const int row = blockIdx.x, chunks = K >> 3;
  const uint16_t* xr = x + (size_t)row * ldx;
  uint4 v[Q8_CHUNKS];
  float amax = 0.f;
#pragma unroll
  for (int u = 0; u < Q8_CHUNKS; ++u) {
    const int c = u * 256 + threadIdx.x;
    v[u] = make_uint4(0u, 0u, 0u, 0u);
    if (c < chunks) v[u] = *(const uint4*)(xr + (size_t)c * 8);
    float f[8];
    unpack8(v[u], f);
#pragma unroll
    for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(f[e]));
  }
  amax = wave_max(amax);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = amax;
  __syncthreads();
  amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  const float s = amax == 0.f ? 1.0f : amax / 448.0f;
  if (threadIdx.x == 0) scale[row] = s;
  uint8_t* qr = q + (size_t)row * ldq;
#pragma unroll
  for (int u = 0; u < Q8_CHUNKS; ++u) {
    const int c = u * 256 + threadIdx.x;
    if (c >= chunks) continue;
    float f[8];
    unpack8(v[u], f);
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = fminf(fmaxf(f[e] / s, -448.0f), 448.0f);
    int w0 = 0, w1 = 0;
    w0 = __builtin_amdgcn_cvt_pk_fp8_f32(f[0], f[1], w0, false);
    w0 = __builtin_amdgcn_cvt_pk_fp8_f32(f[2], f[3], w0, true);
    w1 = __builtin_amdgcn_cvt_pk_fp8_f32(f[4], f[5], w1, false);
    w1 = __builtin_amdgcn_cvt_pk_fp8_f32(f[6], f[7], w1, true);
    *(uint2*)(qr + (size_t)c * 8) = make_uint2((uint32_t)w0, (uint32_t)w1);
  }
}

hipError_t launch_quantize_rows_f8(const void* x, int rows, int K, int ldx, void* q, int ldq,
                                   float* scale, hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  if (K <= 0 || K % 8 != 0 || K > 256 * 8 * Q8_CHUNKS || ldx % 8 != 0 || ldq % 8 != 0 || ldx < K ||
      ldq < K || ((uintptr_t)x & 15) != 0 || ((uintptr_t)q & 7) != 0)
    return hipErrorInvalidValue;
  hipLaunchKernelGGL(quantize_rows_f8_kernel, dim3(rows), dim3(256), 0, st, (const uint16_t*)x, ldx, K,
                     (uint8_t*)q, ldq, scale);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Tile kernel: 256 x 256 tile on 8 waves (4 x 2 waves of 64 x 128; TM = 1: 128 x 256 tile, waves
// of 32 x 128, for launches that would not fill the chip otherwise), 128 K elements (= 128 bytes
// per operand row, the same LDS geometry as the 16-bit kernels) per step, two LDS stages filled
// by global -> LDS copies.  Same ping-pong schedule as the 16-bit kernel: the two waves of a SIMD
// run half a step apart, one in a phase of 8 back-to-back MFMAs (64 cycles each) with the copies
// of the next step riding behind them, the other reading its next fragments from LDS; a bare
// barrier ends every phase.  A lane's fragment of one MFMA is 32 consecutive bytes of its row
// (two 16-byte LDS reads); both operands use the same lane -> k assignment, which is all the
// contraction needs.
// ------------------------------------------------------------------------------------------
constexpr int F8_BK = 128;                          // K elements (bytes) per step

template <int EPI, int TM>
__global__ void __launch_bounds__(512)
gemm_f8_kernel(const uint8_t* __restrict__ A, const uint8_t* __restrict__ W,
               const float* __restrict__ sa, const float* __restrict__ sw,
               uint16_t* __restrict__ C, const uint16_t* __restrict__ R, int M, int N, int K,
               int lda, int ldw, int ldc, int tiles_m, int tiles_n, int group_m, EpiArgs ra) {
  constexpr int NWAVES = 8, WM = 4, WN = 2, TN = 4;
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  constexpr int A_INSTR = BM / 8 / NWAVES, W_INSTR = BN / 8 / NWAVES;    // copies per wave and K step
  constexpr int NCOPY = A_INSTR + W_INSTR;
  constexpr int CPM = (NCOPY + TM * TN - 1) / (TM * TN);                 // copies behind one MFMA
  static_assert((TM == 1 || TM == 2) && NCOPY % CPM == 0 && NCOPY / CPM <= TM * TN, "128- or 256-row tiles");
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
  const int group = wave >> 2;                    // waves w and w+4 share a SIMD

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
    a_off[q] = (uint32_t)((size_t)r * lda + cchunk * 16);
  }
#pragma unroll
  for (int q = 0; q < W_INSTR; ++q) {
    const int tr = (wave * W_INSTR + q) * 8 + crow;
    const int cchunk = (lane & 7) ^ swz64(tr);
    int r = n0 + tr;
    r = r < N ? r : N - 1;
    w_off[q] = (uint32_t)((size_t)r * ldw + cchunk * 16);
  }
  const size_t wstep = (size_t)ra.w_step_bytes;     // 128, or N * 128 for the K-step-major weight
  auto issue = [&](int stage, int k0) {
    char* sal = lds + stage * STAGE_BYTES + (wave * A_INSTR) * 1024;
    char* swl = lds + stage * STAGE_BYTES + BM * ROW_BYTES + (wave * W_INSTR) * 1024;
    const char* gw = (const char*)W + (size_t)(k0 / F8_BK) * wstep;
#pragma unroll
    for (int q = 0; q < A_INSTR; ++q) g2l16((const char*)A + k0 + a_off[q], sal + q * 1024);
#pragma unroll
    for (int q = 0; q < W_INSTR; ++q) g2l16(gw + w_off[q], swl + q * 1024);
  };
  auto issue_one = [&](int stage, int k0, int q) {
    if (q < A_INSTR)
      g2l16((const char*)A + k0 + a_off[q], lds + stage * STAGE_BYTES + (wave * A_INSTR + q) * 1024);
    else
      g2l16((const char*)W + (size_t)(k0 / F8_BK) * wstep + w_off[q - A_INSTR],
            lds + stage * STAGE_BYTES + BM * ROW_BYTES + (wave * W_INSTR + q - A_INSTR) * 1024);
  };

  // fragment of half h (64 K elements) of a row: chunks 4h + 2*(lane >> 5) and the next one
  uint32_t koff[2][2];
#pragma unroll
  for (int h = 0; h < 2; ++h)
#pragma unroll
    for (int u = 0; u < 2; ++u)
      koff[h][u] = (uint32_t)(((4 * h + 2 * (lane >> 5) + u) ^ swz64(lane & 31)) * 16);
  const uint32_t a_row = (uint32_t)((wm * TM * 32 + (lane & 31)) * ROW_BYTES);
  const uint32_t w_row = (uint32_t)(BM * ROW_BYTES + (wn * TN * 32 + (lane & 31)) * ROW_BYTES);

  floatx16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  v8i_t af[TM], wf[TN];

#define LZ_F8_MFMA(i, j)                                                                       \
  acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wf[j], af[i], acc[i][j], 0, 0, 0, 0, 0, 0)
#define LZ_COMPUTE_COPY_PHASE(stage, k0)                                                       \
  do {                                                                                         \
    __builtin_amdgcn_s_setprio(1);                                                             \
    _Pragma("unroll") for (int i = 0; i < TM; ++i)                                             \
      _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                         \
        LZ_F8_MFMA(i, j);                                                                      \
        _Pragma("unroll") for (int cc = 0; cc < CPM; ++cc)                                     \
          if ((i * TN + j) * CPM + cc < NCOPY) issue_one((stage), (k0), (i * TN + j) * CPM + cc); \
      }                                                                                        \
    _Pragma("unroll") for (int n = 0; n < NCOPY / CPM; ++n) {                                  \
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                       \
      __builtin_amdgcn_sched_group_barrier(0x010, CPM, 0);                                     \
    }                                                                                          \
    if (TM * TN > NCOPY / CPM) __builtin_amdgcn_sched_group_barrier(0x008, TM * TN - NCOPY / CPM, 0); \
    __builtin_amdgcn_s_setprio(0);                                                             \
  } while (0)
#define LZ_FRAG(base, h)                                                                       \
  __builtin_shufflevector(*(const v4i_t*)((base) + koff[h][0]), *(const v4i_t*)((base) + koff[h][1]), \
                          0, 1, 2, 3, 4, 5, 6, 7)
#define LZ_MEM_PHASE(st, h)                                                                    \
  do {                                                                                         \
    _Pragma("unroll") for (int i = 0; i < TM; ++i)                                             \
      af[i] = LZ_FRAG((st) + a_row + i * 32 * ROW_BYTES, h);                                   \
    _Pragma("unroll") for (int j = 0; j < TN; ++j)                                             \
      wf[j] = LZ_FRAG((st) + w_row + j * 32 * ROW_BYTES, h);                                   \
  } while (0)
#define LZ_COMPUTE_PHASE()                                                                     \
  do {                                                                                         \
    __builtin_amdgcn_s_setprio(1);                                                             \
    _Pragma("unroll") for (int i = 0; i < TM; ++i)                                             \
      _Pragma("unroll") for (int j = 0; j < TN; ++j) LZ_F8_MFMA(i, j);                         \
    __builtin_amdgcn_s_setprio(0);                                                             \
  } while (0)
  // End of a phase: nothing may be scheduled across it; the barrier is the bare instruction
  // (__syncthreads() would also wait for the copies that were just issued).
#define LZ_PHASE_END()                                                                         \
  do {                                                                                         \
    __builtin_amdgcn_sched_barrier(0);                                                         \
    asm volatile("s_barrier" ::: "memory");                                                    \
    __builtin_amdgcn_sched_barrier(0);                                                         \
  } while (0)

  // NSTAGE LDS stages: the copies of K step t + NSTAGE - 1 are issued while step t computes, so
  // NSTAGE - 1 steps are in flight.  The 128-row tile has room for three stages (48 KB each); it
  // is chosen for launches of few workgroups, where one step in flight per CU (a round trip to
  // HBM per 48 KB) would be the bound.  Waiting for "all but the newest PEND copies" is enough
  // to know that the next step has landed: the counter retires copies in issue order.
  constexpr int NSTAGE = TM == 1 ? 3 : 2;
  constexpr int PEND = (NSTAGE - 2) * NCOPY;
  const int KT = K / F8_BK;
#pragma unroll
  for (int s0 = 0; s0 < NSTAGE - 1; ++s0) issue(s0, (s0 < KT ? s0 : KT - 1) * F8_BK);
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PEND) : "memory");
  __syncthreads();
  if (group == 1) LZ_PHASE_END();                 // the second group starts one phase later
  const bool idle_wave = m0 + wm * TM * 32 >= M;
  int st_cur = 0, st_fill = NSTAGE - 1;
  for (int kt = 0; kt < KT; ++kt) {
    const char* cur = lds + st_cur * STAGE_BYTES;
    // past the last step the copies fetch the last step again, into a stage nobody reads any
    // more (no branch in the MFMA stream; they are drained by the waits like any other)
    const int k_next = (kt + NSTAGE - 1 < KT ? kt + NSTAGE - 1 : KT - 1) * F8_BK;
    if (idle_wave) {                               // all rows past M: copies and barriers only
      LZ_PHASE_END();
#pragma unroll
      for (int q = 0; q < NCOPY; ++q) issue_one(st_fill, k_next, q);
      LZ_PHASE_END();
      if (group == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PEND) : "memory");
      LZ_PHASE_END();
      if (group == 0) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PEND) : "memory");
      LZ_PHASE_END();
    } else {
      LZ_MEM_PHASE(cur, 0);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      LZ_PHASE_END();
      LZ_COMPUTE_COPY_PHASE(st_fill, k_next);
      LZ_PHASE_END();
      LZ_MEM_PHASE(cur, 1);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      if (group == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PEND) : "memory");
      LZ_PHASE_END();
      LZ_COMPUTE_PHASE();
      if (group == 0) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PEND) : "memory");
      LZ_PHASE_END();
    }
    st_cur = st_cur + 1 == NSTAGE ? 0 : st_cur + 1;
    st_fill = st_fill + 1 == NSTAGE ? 0 : st_fill + 1;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); // (the refetches of the last step)
  if (group == 0) LZ_PHASE_END();
#undef LZ_MEM_PHASE
#undef LZ_FRAG
#undef LZ_COMPUTE_PHASE
#undef LZ_COMPUTE_COPY_PHASE
#undef LZ_PHASE_END
#undef LZ_F8_MFMA

  // the operands' scales: one per token row (this lane's TM rows) and one per output feature
  // (register r of block j is feature 8*(r/4) + 4*(lane>>5) + r%4 of the block)
  float sr[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int row = m0 + (wm * TM + i) * 32 + (lane & 31);
    sr[i] = row < M ? sa[row] : 0.f;
  }
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const float* swp = sw + n0 + (wn * TN + j) * 32 + 4 * (lane >> 5);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 c4 = *(const float4*)(swp + 8 * g);
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        acc[i][j][4 * g] *= sr[i] * c4.x;     acc[i][j][4 * g + 1] *= sr[i] * c4.y;
        acc[i][j][4 * g + 2] *= sr[i] * c4.z; acc[i][j][4 * g + 3] *= sr[i] * c4.w;
      }
    }
  }

  if (EPI == EPI_SWIGLU || !ra.stage_out) {
    gemm_epilogue<TM, TN, EPI>(acc, C, R, M, ldc, m0, n0, wm, wn, lane, ra);
    return;
  }
  staged_tile_out<TM, TN, EPI, BM, BN, NWAVES>(acc, C, R, M, ldc, m0, n0, wm, wn, wave, lane, ra, nullptr, lds);
}

hipError_t launch_gemm_f8(const void* A, const float* sa, const void* W, const float* sw, void* C,
                          const void* R, int M, int N, int K, int lda, int ldw, int ldc, int epilogue,
                          hipStream_t st, const EpiArgs* ea_in) {
  constexpr int BN = 256;
  if (M <= 0) return hipSuccess;
  if (N % BN != 0 || K % F8_BK != 0 || lda % 16 != 0 || ldw % 16 != 0 || lda < K || ldw < K ||
      ((uintptr_t)A & 15) != 0 || ((uintptr_t)W & 15) != 0 || ((uintptr_t)sw & 15) != 0)
    return hipErrorInvalidValue;
  if ((size_t)M * lda >= (1ull << 32) || (size_t)N * ldw >= (1ull << 32)) return hipErrorInvalidValue;
  EpiArgs ea{};
  if (ea_in != nullptr) ea = *ea_in;
  if (epilogue == EPI_QKV_ROPE) {
    const int kvd = ea.kv_dim > 0 ? ea.kv_dim : ea.d_model;
    if (ea_in == nullptr || (ea.head_dim != 64 && ea.head_dim != 128) || N != ea.d_model + 2 * kvd)
      return hipErrorInvalidValue;
  }
  // One workgroup per CU is resident.  A launch whose 128-row tiles still fit one round of the
  // 256 CUs takes those (half the K-loop work per workgroup, twice the workgroups); anything
  // larger takes 256-row tiles, which reuse each W slab for twice the rows (measured: gate/up at
  // 2364 rows 214 us against 262 us with 128-row tiles, although the latter need fewer
  // half-rounds).  Every output element sees the same sequence of additions either way.
  const int tiles_n = N / BN;
  const long t128 = (long)((M + 127) / 128) * tiles_n;
  const bool tall = t128 > 256;
  const int BM = tall ? 256 : 128;
  const int LDS_BYTES = (tall ? 2 : 3) * (BM + BN) * ROW_BYTES;
  const int tiles_m = (M + BM - 1) / BM;
  // K-step-major codes ([K / 128][N][128], see launch_pack_kblock): rows of a step 128 bytes apart
  ea.w_step_bytes = ea.w_blocked ? (unsigned long long)N * ROW_BYTES : (unsigned long long)ROW_BYTES;
  if (ea.w_blocked) ldw = F8_BK;
  ea.sf_blocks_per_seq = (ea.sf_max_rows + 511) / 512;
  ea.stage_out = (epilogue == EPI_QKV_ROPE)
                     ? (ea.d_model % BN == 0 && (ea.kv_dim > 0 ? ea.kv_dim : ea.d_model) % BN == 0)
                     : (epilogue != EPI_SWIGLU && ldc % 8 == 0 && ((uintptr_t)C & 15) == 0);
  const int side = ea.sf_z != nullptr ? ea.sf_blocks_per_seq * ea.sf_batch : 0;
  const int band = tall ? 8 : 16;
  const int group_m = tiles_m < band ? tiles_m : band;
  dim3 grid(tiles_m * tiles_n + side), block(512);
#define LZ_GEMM2(E, TMV)                                                                         \
  do {                                                                                           \
    auto kern = gemm_f8_kernel<E, TMV>;                                                          \
    static bool attr_set = false;                                                                \
    if (!attr_set) {                                                                             \
      hipError_t e = hipFuncSetAttribute((const void*)kern,                                      \
                                         hipFuncAttributeMaxDynamicSharedMemorySize,             \
                                         (TMV == 1 ? 3 : 2) * (128 * TMV + BN) * ROW_BYTES);                      \
      if (e != hipSuccess) return e;                                                             \
      attr_set = true;                                                                           \
    }                                                                                            \
    hipLaunchKernelGGL(kern, grid, block, LDS_BYTES, st, (const uint8_t*)A, (const uint8_t*)W,   \
                       sa, sw, (uint16_t*)C, (const uint16_t*)R, M, N, K, lda, ldw, ldc,         \
                       tiles_m, tiles_n, group_m, ea);                                           \
  } while (0)
#define LZ_GEMM(E)                                                                               \
  do {                                                                                           \
    if (tall) LZ_GEMM2(E, 2);                                                                    \
    else LZ_GEMM2(E, 1);                                                                         \
  } while (0)
  if (epilogue == EPI_STORE) LZ_GEMM(EPI_STORE);
  else if (epilogue == EPI_RESIDUAL) LZ_GEMM(EPI_RESIDUAL);
  else if (epilogue == EPI_SWIGLU) LZ_GEMM(EPI_SWIGLU);
  else if (epilogue == EPI_QKV_ROPE) {
    if (ea.head_dim == 64) LZ_GEMM(EPI_QKV_ROPE64);
    else LZ_GEMM(EPI_QKV_ROPE128);
  }
  else return hipErrorInvalidValue;
#undef LZ_GEMM
#undef LZ_GEMM2
  return hipGetLastError();
}

}  // namespace lz
