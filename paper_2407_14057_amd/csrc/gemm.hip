// bf16 GEMM on the gfx950 matrix cores: C[M,N] = A[M,K] W[N,K]^T, fp32 accumulation.
// Both operands are K-contiguous, which is the layout v_mfma_f32_32x32x16_bf16 wants:
// lane l supplies row (l & 31), k elements 8*(l >> 5) .. +8 of a 32x16 operand block.
//
// Workgroup = WM x WN waves, each wave owns TM x TN blocks of 32x32 (fp32 accumulators stay
// in registers for the whole K loop).  K advances 64 elements per step; the A and W slabs of
// a step are copied global -> LDS by global_load_lds (no register staging) into one of two
// LDS stages while the other stage feeds the MFMAs.
//
// W may be row-major [N][K] (row stride ldw) or K-step-major [K/64][N][64] (EpiArgs::w_blocked, the
// order the model keeps its weights in): the kernels only differ in two byte strides, row to row
// (ldw * 2 or 128) and K step to K step (128 or N * 128).  K-step-major, the slab of one step is
// one contiguous run, which the memory system serves better than one line from each of 256 rows.
#include <stdlib.h>

#include "common.h"
#include "gemm_shared.h"

namespace lz {

// Workspace of the forms that exchange partial sums between workgroups.  Layout: fp32 partial tiles
// (64 MB) | 4 KB of tickets of the skinny kernel (see gemm_skinny_kernel) | 4 KB of flags of the
// persistent stream-K kernel (see gemm_psk_kernel), of which words 1008..1016 are the tile
// counters of the ping-pong kernel's tile walk (see gemm_pp_kernel).  Tickets, flags and counters
// must be zero before the first launch that uses them; every launch leaves them zero again.
constexpr int SK_GRID = 512;
constexpr size_t SK_PART_BYTES = (size_t)SK_GRID * 2 * 128 * 128 * sizeof(float);
constexpr size_t SK_TICKET_BYTES = 4096, PSK_FLAG_BYTES = 4096;
constexpr int PSK_FLAG_WORDS_MAX = 1000, WALK_TICKET_WORD = 1008;      // (word 1023 counts the stream-K give-ups)

template <int WM, int WN, int TM, int TN, int EPI, int NS = 2>
__global__ void __launch_bounds__(WM * WN * 64)
gemm_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ W,
            uint16_t* __restrict__ C, const uint16_t* __restrict__ R, int M, int N, int K, int lda,
            int ldw, int ldc, int tiles_m, int tiles_n, int group_m, EpiArgs ra) {
  constexpr int NWAVES = WM * WN;
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  constexpr int A_INSTR = BM / 8 / NWAVES;      // wave-wide 1 KB copies per wave per step
  constexpr int W_INSTR = BN / 8 / NWAVES;
  constexpr int STAGE_BYTES = (BM + BN) * ROW_BYTES;
  static_assert(BM % (8 * NWAVES) == 0 && BN % (8 * NWAVES) == 0, "tile/wave mismatch");
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

  // ---- workgroup -> tile.  Consecutive workgroup ids land on different XCDs (8 of them,
  // each with its own L2), so ids are first regrouped per XCD, then walked in bands of
  // GROUP_M tile rows so that concurrently running tiles share A and W slabs in L2.
  int tile_m, tile_n;
  workgroup_tile((int)blockIdx.x, tiles_m, tiles_n, group_m, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  // ---- global -> LDS copy plan.  Lane p of a wave instruction fills LDS bytes
  // [16p, 16p+16) of an 8-row slab: row p/8, stored chunk p%8, which holds logical
  // chunk (p%8) ^ swz64(row).
  const int crow = lane >> 3;
  uint32_t a_off[A_INSTR], w_off[W_INSTR];
#pragma unroll
  for (int q = 0; q < A_INSTR; ++q) {
    const int tr = (wave * A_INSTR + q) * 8 + crow;          // row inside the tile
    const int cchunk = (lane & 7) ^ swz64(tr);
    int r = m0 + tr;
    r = r < M ? r : M - 1;                       // rows past the edge: re-read the last row
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

  const size_t wstep = (size_t)ra.w_step_bytes;     // 128, or N * 128 for the K-step-major weight
  auto issue = [&](int stage, int k0) {
    char* sa = lds + stage * STAGE_BYTES + (wave * A_INSTR) * 1024;
    char* sw = lds + stage * STAGE_BYTES + BM * ROW_BYTES + (wave * W_INSTR) * 1024;
    const char* ga = (const char*)A + (size_t)k0 * 2;
    const char* gw = (const char*)W + (size_t)(k0 / BK) * wstep;
#pragma unroll
    for (int q = 0; q < A_INSTR; ++q) g2l16(ga + a_off[q], sa + q * 1024);
#pragma unroll
    for (int q = 0; q < W_INSTR; ++q) g2l16(gw + w_off[q], sw + q * 1024);
  };

  // ---- MFMA operand addresses: row (l & 31) of a 32-row block, chunk 2*ks + (l >> 5)
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

  // ---- main loop.  Operand fragments are double-buffered in registers: the reads for k-step
  // s+1 are issued before the MFMAs of k-step s.  The single barrier of an iteration sits
  // before the last k-step, when every wave has pulled its last fragments of the current
  // stage into registers; the stage is then free to receive the tile two steps ahead, and the
  // first fragments of the next stage are fetched under the last 16 MFMAs.
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
  // Order inside a k-step: the LDS reads of the NEXT k-step go out first, one or two per MFMA,
  // so that the last of them still has at least half a k-step of MFMAs to land under.
#define LZ_SCHED()                                                                            \
  do {                                                                                        \
    constexpr int NR = TM + TN, NM = TM * TN;                                                 \
    constexpr int RPG = (NR * 2 > NM) ? 2 : 1;          /* reads per group */                 \
    constexpr int NG = NR / RPG;                                                              \
    _Pragma("unroll") for (int n = 0; n < NG; ++n) {                                          \
      __builtin_amdgcn_sched_group_barrier(0x100, RPG, 0);                                    \
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                      \
    }                                                                                         \
    __builtin_amdgcn_sched_group_barrier(0x008, NM - NG, 0);                                  \
  } while (0)

  // NS stages: K step kt lives in stage kt mod NS; steps 0 .. NS-1 are copied up front, step
  // kt + NS in iteration kt, right after the barrier that frees step kt's stage.  With more than
  // two stages the barrier waits only for the copies of step kt + 1 (everything but the newest
  // NS - 2 steps' worth): a copy then has NS - 3/4 iterations to arrive instead of 1 1/4.
  static_assert(NS == 2 || NS == 3, "two or three stages");
  const int KT = K / BK;
#pragma unroll
  for (int t = 0; t < NS; ++t)
    if (t < KT) issue(t, t * BK);
  float rs[TM];
  load_row_scales<TM>(rs, ra, M, m0, wm, lane);
  // (three steps in flight: only the first has to be there; the row scales fetched last are needed in the epilogue)
  if (NS == 3 && KT >= 3) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 1) * (A_INSTR + W_INSTR)) : "memory");
  else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  LZ_LOAD_FRAGS(0, lds, 0);
  int st_cur = 0;                                   // kt mod NS
  for (int kt = 0; kt < KT; ++kt) {
    const int st_nxt = st_cur + 1 == NS ? 0 : st_cur + 1;
    const char* cur = lds + st_cur * STAGE_BYTES;
    const char* nxt = lds + st_nxt * STAGE_BYTES;
    LZ_LOAD_FRAGS(1, cur, 1);
    LZ_MFMAS(0);
    LZ_SCHED();
    LZ_LOAD_FRAGS(0, cur, 2);
    LZ_MFMAS(1);
    LZ_SCHED();
    LZ_LOAD_FRAGS(1, cur, 3);
    LZ_MFMAS(0);
    LZ_SCHED();
    // step kt + 1 must have landed; with three stages step kt + 2 (issued an iteration ago) may
    // still be on its way, unless it does not exist
    if (NS == 3 && kt + 2 < KT) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(A_INSTR + W_INSTR) : "memory");
    else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __syncthreads();
    if (kt + NS < KT) issue(st_cur, (kt + NS) * BK);
    if (kt + 1 < KT) LZ_LOAD_FRAGS(0, nxt, 0);
    LZ_MFMAS(1);
    LZ_SCHED();
    st_cur = st_nxt;
  }
#undef LZ_LOAD_FRAGS
#undef LZ_MFMAS
#undef LZ_SCHED

  gemm_epilogue<TM, TN, EPI>(acc, C, R, M, ldc, m0, n0, wm, wn, lane, ra, rs);
}

template <int WM, int WN, int TM, int TN, int NS = 2>
static hipError_t launch_cfg(const void* A, const void* W, void* C, const void* R, int M, int N,
                             int K, int lda, int ldw, int ldc, int epi, int group_m,
                             const EpiArgs& ra, hipStream_t st) {
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  constexpr int LDS_BYTES = NS * (BM + BN) * ROW_BYTES;
  static_assert(LDS_BYTES <= 160 * 1024, "LDS of a CU");
  if (N % BN != 0) return hipErrorInvalidValue;
  const int tiles_m = (M + BM - 1) / BM, tiles_n = N / BN;
  const int threads = WM * WN * 64;
  EpiArgs ea = ra;
  ea.w_step_bytes = ra.w_blocked ? (unsigned long long)N * ROW_BYTES : (unsigned long long)ROW_BYTES;
  if (ra.w_blocked) ldw = BK;                       // rows of one K step are 128 bytes apart
  ea.sf_blocks_per_seq = (ea.sf_max_rows + threads - 1) / threads;
  const int side = ea.sf_z != nullptr ? ea.sf_blocks_per_seq * ea.sf_batch : 0;
  dim3 grid(tiles_m * tiles_n + side), block(threads);
#define LZ_GEMM(E)                                                                               \
  do {                                                                                           \
    auto kern = gemm_kernel<WM, WN, TM, TN, E, NS>;                                              \
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
    if ((TN * 32) % ra.head_dim != 0) return hipErrorInvalidValue;
    if (ra.head_dim == 64) LZ_GEMM(EPI_QKV_ROPE64);
    else if constexpr (TN >= 4) LZ_GEMM(EPI_QKV_ROPE128);
    else return hipErrorInvalidValue;
  }
  else return hipErrorInvalidValue;
#undef LZ_GEMM
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Ping-pong kernel on 8 waves: the 256x256x64 tile as 4 x 2 waves of 64 x 128, or the 192x256x64
// tile as 2 x 4 waves of 96 x 64 (the figures below are for the first).  The two
// waves that share a SIMD (wave w and w + 4) run the same loop half a step apart: while one
// is in a COMPUTE phase (16 back-to-back MFMAs, nothing else), the other is in a MEMORY phase
// (the 12 LDS reads of its next half step, its global -> LDS copies, the waits).  A workgroup
// barrier closes every phase, so the matrix pipe of each SIMD always has exactly one wave
// feeding it and that wave's instruction stream is pure MFMA.
//   phase p:      0      1      2      3      4    ...
//   waves 0-3:   M(0a)  C(0a)  M(0b)  C(0b)  M(1a) ...       a, b = first / second half of a
//   waves 4-7:    -     M(0a)  C(0a)  M(0b)  C(0b) ...              64-wide K step
// The global -> LDS copies are issued from COMPUTE phases, one after each of the first eight
// MFMAs: the matrix pipe accepts a new MFMA only every 32 cycles, so the copies ride in issue
// slots that are idle anyway, whereas in front of the LDS reads of a memory phase they delay
// those reads and make the memory phase the longer one (measured: 1.69 vs 1.30 PFLOP/s in a
// loop of this shape).  The stage of K step t is last read in phase 4t+3 and step t+1 is first
// read in phase 4t+4, so every wave copies its share of step t+1 during C(t a) (phases 4t+1 and
// 4t+2) and waits for it before the barrier that ends phase 4t+3.
// ------------------------------------------------------------------------------------------
template <int WM, int WN, int TM, int TN, int EPI>
__global__ void __launch_bounds__(512)
gemm_pp_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ W,
               uint16_t* __restrict__ C, const uint16_t* __restrict__ R, int M, int N, int K,
               int lda, int ldw, int ldc, int tiles_m, int tiles_n, int group_m, EpiArgs ra) {
  constexpr int NWAVES = 8;
  static_assert(WM * WN == NWAVES, "eight waves: two per SIMD");
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  constexpr int A_INSTR = BM / 8 / NWAVES, W_INSTR = BN / 8 / NWAVES;    // copies per wave and K step
  constexpr int NCOPY = A_INSTR + W_INSTR;
  static_assert(BM % 64 == 0 && BN % 64 == 0 && NCOPY <= 2 * TM * TN, "tile/wave mismatch");
  constexpr int STAGE_BYTES = (BM + BN) * ROW_BYTES;
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  // The SiLU*mul form walks its tiles when there are more tiles than compute units: `ra.pp_walkers`
  // workgroups, one per CU, start on tiles 0 .. walkers-1 and then draw further tiles from a
  // counter of their XCD (tiles walkers + x + 8n for XCD x, in order: the CUs of an XCD keep
  // working on neighbouring tiles, as under the dispatcher, and a CU that runs ahead takes more).
  // A tile's last K step copies step 0 of the NEXT tile (in the slot where a tile of its own
  // launch re-copies its last step for nothing), so the next tile starts without a first-load
  // latency, and the tile's stores drain behind the next tile's K loop instead of in front of the
  // next workgroup's start.  The ticket for the next tile is drawn when a tile starts, handed to
  // the other waves through LDS at the end of the first K step and read in the last (so K spans
  // at least two steps); the last workgroup to leave zeroes the counters for the next launch.
  // (The other epilogues need both LDS stages for the tile and stay one tile per workgroup.)
  constexpr bool PERSIST = (EPI == EPI_SWIGLU);
  const int T = tiles_m * tiles_n;
  const int walkers = PERSIST ? ra.pp_walkers : T;
  unsigned* const tk = PERSIST ? ra.walk_tickets : nullptr;   // 8 counters + 1 of leavers; null: no walk
  if ((int)blockIdx.x >= walkers) {               // side job (see EpiArgs): Eq. 1 scores
    const int sb = (int)blockIdx.x - walkers;
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
  int m0 = tile_m * BM, n0 = tile_n * BN;

  const int crow = lane >> 3;
  uint32_t a_off[A_INSTR], w_off[W_INSTR];
  auto set_offsets = [&](int m0_, int n0_) {
#pragma unroll
    for (int q = 0; q < A_INSTR; ++q) {
      const int tr = (wave * A_INSTR + q) * 8 + crow;
      const int cchunk = (lane & 7) ^ swz64(tr);
      int r = m0_ + tr;
      r = r < M ? r : M - 1;
      if (ra.a_rows != nullptr) r = ra.a_rows[r];
      a_off[q] = (uint32_t)(((size_t)r * lda + cchunk * 8) * 2);
    }
#pragma unroll
    for (int q = 0; q < W_INSTR; ++q) {
      const int tr = (wave * W_INSTR + q) * 8 + crow;
      const int cchunk = (lane & 7) ^ swz64(tr);
      int r = n0_ + tr;
      r = r < N ? r : N - 1;
      w_off[q] = (uint32_t)(((size_t)r * ldw + cchunk * 8) * 2);
    }
  };
  set_offsets(m0, n0);
  const size_t wstep = (size_t)ra.w_step_bytes;     // 128, or N * 128 for the K-step-major weight
  auto issue = [&](int stage, int k0) {
    char* sa = lds + stage * STAGE_BYTES + (wave * A_INSTR) * 1024;
    char* sw = lds + stage * STAGE_BYTES + BM * ROW_BYTES + (wave * W_INSTR) * 1024;
    const char* ga = (const char*)A + (size_t)k0 * 2;
    const char* gw = (const char*)W + (size_t)(k0 / BK) * wstep;
#pragma unroll
    for (int q = 0; q < A_INSTR; ++q) g2l16(ga + a_off[q], sa + q * 1024);
#pragma unroll
    for (int q = 0; q < W_INSTR; ++q) g2l16(gw + w_off[q], sw + q * 1024);
  };
  // one of the wave's copies of a K step (q < A_INSTR: A rows, else W rows)
  // (uniform base + 32-bit lane offset: the K step's share of the address then lives in scalar
  // registers and a copy costs the MFMA stream a load and an M0 update, no vector arithmetic --
  // 0.5-3 % per launch against 64-bit lane addresses; the launcher checks that both operands span
  // less than 4 GB)
  const uint32_t wstep32 = (uint32_t)wstep;
  auto issue_one = [&](int stage, int k0, int q) {
    if (q < A_INSTR)
      g2l16((const char*)A + (uint32_t)(a_off[q] + (uint32_t)k0 * 2u),
            lds + stage * STAGE_BYTES + (wave * A_INSTR + q) * 1024);
    else
      g2l16((const char*)W + (uint32_t)(w_off[q - A_INSTR] + (uint32_t)(k0 / BK) * wstep32),
            lds + stage * STAGE_BYTES + BM * ROW_BYTES + (wave * W_INSTR + q - A_INSTR) * 1024);
  };

  uint32_t koff[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
    koff[ks] = (uint32_t)(((ks * 2 + (lane >> 5)) ^ swz64(lane & 31)) * 16);
  const uint32_t a_row = (uint32_t)((wm * TM * 32 + (lane & 31)) * ROW_BYTES);
  const uint32_t w_row = (uint32_t)(BM * ROW_BYTES + (wn * TN * 32 + (lane & 31)) * ROW_BYTES);

  floatx16_t acc[TM][TN];
  bf16x8_t af[2][TM], wf[2][TN];

  // 2*TM*TN MFMAs with one copy behind each of the first NCOPY
#define LZ_COMPUTE_COPY_PHASE(stage, k0)                                                       \
  do {                                                                                         \
    __builtin_amdgcn_s_setprio(1);                                                             \
    _Pragma("unroll") for (int k2 = 0; k2 < 2; ++k2)                                           \
      _Pragma("unroll") for (int i = 0; i < TM; ++i)                                           \
        _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                       \
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[k2][j], af[k2][i], acc[i][j], \
                                                              0, 0, 0);                        \
          if ((k2 * TM + i) * TN + j < NCOPY) issue_one((stage), (k0), (k2 * TM + i) * TN + j); \
        }                                                                                      \
    _Pragma("unroll") for (int n = 0; n < NCOPY; ++n) {                                        \
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                       \
      __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);                                       \
    }                                                                                          \
    __builtin_amdgcn_sched_group_barrier(0x008, 2 * TM * TN - NCOPY, 0);                       \
    __builtin_amdgcn_s_setprio(0);                                                             \
  } while (0)

#define LZ_MEM_PHASE(st, h)                                                                    \
  do {                                                                                         \
    _Pragma("unroll") for (int k2 = 0; k2 < 2; ++k2) {                                         \
      _Pragma("unroll") for (int i = 0; i < TM; ++i)                                           \
        af[k2][i] = *(const bf16x8_t*)((st) + a_row + i * 32 * ROW_BYTES + koff[2 * (h) + k2]); \
      _Pragma("unroll") for (int j = 0; j < TN; ++j)                                           \
        wf[k2][j] = *(const bf16x8_t*)((st) + w_row + j * 32 * ROW_BYTES + koff[2 * (h) + k2]); \
    }                                                                                          \
  } while (0)
#define LZ_COMPUTE_PHASE()                                                                     \
  do {                                                                                         \
    __builtin_amdgcn_s_setprio(1);                                                             \
    _Pragma("unroll") for (int k2 = 0; k2 < 2; ++k2)                                           \
      _Pragma("unroll") for (int i = 0; i < TM; ++i)                                           \
        _Pragma("unroll") for (int j = 0; j < TN; ++j)                                         \
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[k2][j], af[k2][i], acc[i][j], \
                                                              0, 0, 0);                        \
    __builtin_amdgcn_s_setprio(0);                                                             \
  } while (0)
  // End of a phase: nothing may be scheduled across it.  The barrier is the bare instruction:
  // __syncthreads() would also drain vmcnt, i.e. wait for the copies that were just issued and
  // have a whole K step to land; the waits that ARE needed are written out at each phase end.
#define LZ_PHASE_END()                                                                         \
  do {                                                                                         \
    __builtin_amdgcn_sched_barrier(0);                                                         \
    asm volatile("s_barrier" ::: "memory");                                                    \
    __builtin_amdgcn_sched_barrier(0);                                                         \
  } while (0)

  // thread 0 (first group: its wait for the copies, just before, has also brought the ticket in)
  // leaves the drawn ticket in LDS for everybody, a barrier before anyone reads it
  // (instructions written out: the atomic's return must not be waited for where it is issued --
  // the compiler would turn it into a wave-wide reduction with a wait -- and the slot is plain LDS)
  const uint32_t ticket_slot =
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds + 2u * STAGE_BYTES;
#define LZ_HAND_TICKET()                                                                       \
  do {                                                                                         \
    if (PERSIST && tk != nullptr && kt == 0 && threadIdx.x == 0)                               \
      asm volatile("ds_write_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" ::"v"(ticket_slot), "v"(ticket) : "memory"); \
  } while (0)

  const int KT = K / BK;
  issue(0, 0);
  float rs[TM];
  load_row_scales<TM>(rs, ra, M, m0, wm, lane);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  int par = 0;                                    // stage that holds step 0 of the current tile
  for (;;) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    unsigned ticket = 0;
    if (PERSIST && tk != nullptr && threadIdx.x == 0)
      asm volatile("global_atomic_add %0, %1, %2, off sc0"
                   : "=&v"(ticket) : "v"(tk + ((int)blockIdx.x & 7)), "v"(1u) : "memory");
    bool has_next = false;
    int m0_next = 0, n0_next = 0;
    unsigned long long ssq_next[TM];              // row scales of the next tile, as loaded
#pragma unroll
    for (int i = 0; i < TM; ++i) ssq_next[i] = 0;
    if (group == 1) LZ_PHASE_END();               // the second group starts one phase later
    const bool idle_wave = m0 + wm * TM * 32 >= M;
    for (int kt = 0; kt < KT; ++kt) {
      const char* cur = lds + ((kt + par) & 1) * STAGE_BYTES;
      const int st_next = (kt + 1 + par) & 1;
      // The last step copies itself again into the stage nobody reads any more (no branch in
      // the MFMA stream, and the copy is drained by the waits below like any other) -- or, when
      // the workgroup has another tile, that tile's step 0.
      int k_next = (kt + 1 < KT ? kt + 1 : kt) * BK;
      if (PERSIST && tk != nullptr && kt == KT - 1) {
        int drawn;
        asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(drawn) : "v"(ticket_slot) : "memory");
        drawn = __builtin_amdgcn_readfirstlane(drawn);
        const int pid_next = walkers + ((int)blockIdx.x & 7) + 8 * drawn;
        has_next = pid_next < T;
        if (has_next) {
          workgroup_tile(pid_next, tiles_m, tiles_n, group_m, tile_m, tile_n);
          m0_next = tile_m * BM;
          n0_next = tile_n * BN;
          set_offsets(m0_next, n0_next);
          k_next = 0;
          if (ra.ssq_in != nullptr) {             // (used after the loop: nobody waits for it here)
#pragma unroll
            for (int i = 0; i < TM; ++i) {
              const int row = m0_next + (wm * TM + i) * 32 + (lane & 31);
              const int rc = row < M ? row : M - 1;
              ssq_next[i] = ra.ssq_in[ra.a_rows != nullptr ? ra.a_rows[rc] : rc];
            }
          }
        }
      }
      if (idle_wave) {
        // all of this wave's rows are past M (last tile row): it still copies its share of the
        // stages and keeps the barriers, but runs no MFMA -- the part is power-limited, and the
        // matrix work on padding rows would only lower the clock for everybody else
        LZ_PHASE_END();
#pragma unroll
        for (int q = 0; q < NCOPY; ++q) issue_one(st_next, k_next, q);
        LZ_PHASE_END();
        if (group == 1) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        LZ_PHASE_END();
        if (group == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        LZ_HAND_TICKET();
        LZ_PHASE_END();
        continue;
      }
      LZ_MEM_PHASE(cur, 0);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      LZ_PHASE_END();
      LZ_COMPUTE_COPY_PHASE(st_next, k_next);
      LZ_PHASE_END();
      LZ_MEM_PHASE(cur, 1);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      if (group == 1) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      LZ_PHASE_END();
      LZ_COMPUTE_PHASE();
      if (group == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      LZ_HAND_TICKET();
      LZ_PHASE_END();
    }
    if (group == 0) LZ_PHASE_END();
    if (!PERSIST) break;
    // One stage already holds the next tile's step 0; the other one -- the last step's, which
    // nobody reads any more and which step 1 of the next tile overwrites only after that tile's
    // first barrier -- is exactly the size of the SiLU*mul tile (half as wide as the product),
    // so the tile still goes out through LDS in whole rows.
    if (ra.stage_out) {
      static_assert(BM * (BN / 2) * 2 <= STAGE_BYTES, "the SiLU*mul tile must fit one stage");
      staged_tile_out<TM, TN, EPI, BM, BN, NWAVES>(acc, C, R, M, ldc, m0, n0, wm, wn, wave, lane, ra, rs,
                                                   lds + ((KT - 1 + par) & 1) * STAGE_BYTES);
    } else {
      gemm_epilogue<TM, TN, EPI>(acc, C, R, M, ldc, m0, n0, wm, wn, lane, ra, rs);
    }
    if (!has_next) {
      if (tk != nullptr && threadIdx.x == 0) {
        const unsigned left = __hip_atomic_fetch_add(tk + 8, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (left == (unsigned)walkers - 1u)         // everybody else has drawn their last ticket
          for (int x = 0; x < 9; ++x) __hip_atomic_store(tk + x, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      return;
    }
    m0 = m0_next;
    n0 = n0_next;
    par = (par + KT) & 1;
#pragma unroll
    for (int i = 0; i < TM; ++i)
      rs[i] = (ra.ssq_in != nullptr && m0 + (wm * TM + i) * 32 + (lane & 31) < M)
                  ? rsqrtf((float)ssq_next[i] * ra.ssq_mul + ra.eps) : 0.f;
  }
#undef LZ_MEM_PHASE
#undef LZ_COMPUTE_PHASE
#undef LZ_COMPUTE_COPY_PHASE
#undef LZ_PHASE_END
#undef LZ_HAND_TICKET
  if (!ra.stage_out) {
    gemm_epilogue<TM, TN, EPI>(acc, C, R, M, ldc, m0, n0, wm, wn, lane, ra, rs);
    return;
  }
  static_assert(BM * BN * 2 <= 2 * STAGE_BYTES, "staged tile must fit the stages");
  staged_tile_out<TM, TN, EPI, BM, BN, NWAVES>(acc, C, R, M, ldc, m0, n0, wm, wn, wave, lane, ra, rs, lds);
}

// Workgroups of a persistent kernel that are resident at once (one per CU when the device is
// otherwise idle); 0 if the runtime cannot tell.
template <typename KernT>
static int psk_resident_workgroups(KernT kern, int lds_bytes) {
  int dev = 0, per_cu = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)kern, 512, (size_t)lds_bytes) != hipSuccess)
    return 0;
  return per_cu >= 1 ? cus : 0;
}

// The ping-pong kernels address both operands with 32-bit byte offsets from a uniform base.
static bool pp_operands_fit_32bit(int M, int N, int K, int lda, int ldw, bool w_blocked) {
  return (unsigned long long)M * lda * 2 < (1ull << 32) &&
         (unsigned long long)N * (w_blocked ? K : ldw) * 2 < (1ull << 32);
}

template <int WM, int WN, int TM, int TN>
static hipError_t launch_pp(const void* A, const void* W, void* C, const void* R, int M, int N,
                            int K, int lda, int ldw, int ldc, int epi, int group_m,
                            const EpiArgs& ra, hipStream_t st) {
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  constexpr int LDS_BYTES = 2 * (BM + BN) * ROW_BYTES + 16;      // two stages and the ticket slot
  if (N % BN != 0) return hipErrorInvalidValue;
  if (!pp_operands_fit_32bit(M, N, K, lda, ldw, ra.w_blocked != 0)) return hipErrorInvalidValue;
  const int tiles_m = (M + BM - 1) / BM, tiles_n = N / BN;
  EpiArgs ea = ra;
  ea.w_step_bytes = ra.w_blocked ? (unsigned long long)N * ROW_BYTES : (unsigned long long)ROW_BYTES;
  if (ra.w_blocked) ldw = BK;                       // rows of one K step are 128 bytes apart
  ea.sf_blocks_per_seq = (ea.sf_max_rows + 511) / 512;
  // the tile goes out through LDS when whole 16-byte chunks of every row are addressable
  ea.stage_out = (epi == EPI_QKV_ROPE) ? (ra.d_model % BN == 0 && (ra.kv_dim > 0 ? ra.kv_dim : ra.d_model) % BN == 0)
                 : (ldc % 8 == 0 && ((uintptr_t)C & 15) == 0);
  const int side = ea.sf_z != nullptr ? ea.sf_blocks_per_seq * ea.sf_batch : 0;
  dim3 block(512);
#define LZ_GEMM(E)                                                                               \
  do {                                                                                           \
    auto kern = gemm_pp_kernel<WM, WN, TM, TN, E>;                                               \
    static bool attr_set = false;                                                                \
    static int resident = 0;                                                                     \
    if (!attr_set) {                                                                             \
      hipError_t e = hipFuncSetAttribute((const void*)kern,                                      \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES); \
      if (e != hipSuccess) return e;                                                             \
      resident = psk_resident_workgroups(kern, LDS_BYTES);                                       \
      attr_set = true;                                                                           \
    }                                                                                            \
    /* the SiLU*mul form walks its tiles with one workgroup per CU (a whole number per XCD) when \
       it has the ticket counters; every other form: one workgroup per tile */                   \
    const int cus = resident & ~7;                                                               \
    const bool walk = E == EPI_SWIGLU && ra.walk_tickets != nullptr && cus >= 8 &&               \
                      cus < tiles_m * tiles_n && K >= 2 * BK;                                    \
    ea.pp_walkers = walk ? cus : tiles_m * tiles_n;                                              \
    if (!walk) ea.walk_tickets = nullptr;                                                        \
    dim3 grid(ea.pp_walkers + side);                                                             \
    hipLaunchKernelGGL(kern, grid, block, LDS_BYTES, st, (const uint16_t*)A, (const uint16_t*)W, \
                       (uint16_t*)C, (const uint16_t*)R, M, N, K, lda, ldw, ldc, tiles_m,        \
                       tiles_n, group_m, ea);                                                    \
  } while (0)
  if (epi == EPI_STORE) LZ_GEMM(EPI_STORE);
  else if (epi == EPI_RESIDUAL) LZ_GEMM(EPI_RESIDUAL);
  else if (epi == EPI_SWIGLU) LZ_GEMM(EPI_SWIGLU);
  else if (epi == EPI_QKV_ROPE) {
    if (ra.head_dim == 64) LZ_GEMM(EPI_QKV_ROPE64);
    else if constexpr (TN >= 4) LZ_GEMM(EPI_QKV_ROPE128);
    else return hipErrorInvalidValue;
  }
  else return hipErrorInvalidValue;
#undef LZ_GEMM
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Persistent stream-K form of the ping-pong kernel.  A data-parallel launch runs ceil(T / 256)
// rounds of tiles on 256 CUs however few tiles the last round holds (1204 tiles: 5 rounds for
// 4.7 rounds of work; 160 tiles: one round on 62 % of the chip).  Here G workgroups, one per CU
// and all resident at once, each take an equal share of the work:
//   * the first floor(T / G) * G tiles run data-parallel, workgroup g taking tiles g, g + G, ...
//     (same tile walk as the data-parallel kernel, so the L2 sharing is unchanged);
//   * the K steps of the remaining Rm < G tiles, U = Rm * KT units, are cut into G equal
//     contiguous ranges.  A range is shorter than a tile, so it covers the END of one tile
//     (the workgroup that holds a tile's last K steps OWNS the tile) and/or the START or a
//     middle piece of the next (a piece it does not own).
// Order inside a workgroup: its data-parallel tiles first (all workgroups of an XCD then walk K in
// step and share operand slabs through the L2, which a head start of a few K steps would undo),
// then the piece it does not own -- a tile's first K steps, so these start together at K = 0;
// the fp32 partial sums go to the workspace, lane-major, 16 bytes per lane and store, followed by
// a flag once they have reached the L2 -- and its own piece LAST: these end together at K = KT,
// and the other pieces of the tile were finished before the owner is (every workgroup gives its
// piece away before it starts its own).  The owner adds them in ascending K order (a fixed order:
// results do not depend on timing) and runs the normal epilogue.  The pieces of a tile belong to
// workgroups of one XCD (ids x, x + 8, ...), which share an L2, so the exchange needs no cache
// write-back or invalidation; that the dispatcher did put them on one XCD is checked, not
// assumed: the flag's value is 1 + the writer's XCC id (hardware register XCC_ID) and the owner
// compares it with its own.  Waits are bounded: if a flag never comes (it cannot, unless fewer
// than G workgroups fit on the device, which the launcher checks) or comes from another XCD,
// the owner gives up, counts the failure in the last word of the flag area -- the prefill and the
// decoding step turn a count into LAZYLLM_ST_EXCHANGE of their status word -- and finishes.
// Flags are zero on entry; the owner resets the flags it consumed.
// ------------------------------------------------------------------------------------------
constexpr unsigned PSK_SPIN_LIMIT = 1u << 22;      // about a second of polling

template <int WM, int WN, int TM, int TN, int EPI>
__global__ void __launch_bounds__(512)
gemm_psk_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ W,
                uint16_t* __restrict__ C, const uint16_t* __restrict__ R, int M, int N, int K,
                int lda, int ldw, int ldc, int tiles_m, int tiles_n, int group_m, int G,
                float* __restrict__ part, unsigned* __restrict__ flags, EpiArgs ra) {
  constexpr int NWAVES = 8;
  static_assert(WM * WN == NWAVES, "eight waves: two per SIMD");
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  constexpr int A_INSTR = BM / 8 / NWAVES, W_INSTR = BN / 8 / NWAVES;
  constexpr int NCOPY = A_INSTR + W_INSTR;
  static_assert(BM % 64 == 0 && BN % 64 == 0 && NCOPY <= 2 * TM * TN, "tile/wave mismatch");
  constexpr int STAGE_BYTES = (BM + BN) * ROW_BYTES;
  constexpr int TILE_FLOATS = BM * BN;
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  __shared__ unsigned wait_failed;
  // the XCC (XCD) this workgroup runs on: hardware register XCC_ID, bits 3:0
  const unsigned my_xcc = __builtin_amdgcn_s_getreg((3 << 11) | (0 << 6) | 20);
  if ((int)blockIdx.x >= G) {                     // side job (see EpiArgs): Eq. 1 scores
    const int sb = (int)blockIdx.x - G;
    score_finish_block<true>(ra.sf_z, ra.sf_stat, ra.sf_s, ra.sf_cu, ra.sf_n_single, ra.sf_heads,
                             ra.sf_z_ld, ra.sf_cu_z, true, sb / ra.sf_blocks_per_seq,
                             (sb % ra.sf_blocks_per_seq) * (int)blockDim.x, (float2*)lds);
    return;
  }

  // `lane` is passed through an empty asm at the start of every section below: the compiler then
  // cannot keep per-lane values of one section (epilogue addresses, say) alive across the K loop
  // of another, which cost the loops their registers (spills that wait behind the tile copies)
  int lane = threadIdx.x & 63;
#define LZ_FRESH_LANE() asm volatile("" : "+v"(lane))
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int group = wave >> 2;                    // waves w and w+4 share a SIMD
  const int g = (int)blockIdx.x;

  // ---- this workgroup's share.  The remainder tiles are split XCD by XCD: workgroup ids are dealt
  // round-robin over the 8 XCDs and the tile walk gives XCD x the tiles whose id is x mod 8, so
  // the G / 8 workgroups of an XCD cut up the K steps of THAT XCD's remainder tiles: neighbours in
  // the walk keep sharing operand slabs through their L2, as in the data-parallel rounds.
  const int T = tiles_m * tiles_n, KT = K / BK;
  const int full = T / G, Rm = T - full * G;
  const int xcd = g & 7, gi = g >> 3, GX = G >> 3;
  const int Rx = Rm > xcd ? (Rm - xcd + 7) >> 3 : 0;           // remainder tiles of this XCD
  const long long U = (long long)Rx * KT;
  auto ubegin = [&](int i) { return (long long)i * U / GX; };   // first unit of the XCD's i-th workgroup
  auto sk_pid = [&](int t) { return full * G + xcd + 8 * t; };  // tile id of the XCD's t-th remainder tile
  const long long u0 = ubegin(gi), u1 = ubegin(gi + 1);
  int own_tile = -1, own_ka = 0, oth_tile = -1, oth_ka = 0, oth_kb = 0;
  if (u1 > u0) {
    const int ta = (int)(u0 / KT), tb = (int)((u1 - 1) / KT);
    if (ta == tb) {
      if (u1 == (long long)(ta + 1) * KT) { own_tile = ta; own_ka = (int)(u0 - (long long)ta * KT); }
      else { oth_tile = ta; oth_ka = (int)(u0 - (long long)ta * KT); oth_kb = (int)(u1 - (long long)ta * KT); }
    } else {                                      // the end of tile ta and the start of tile ta + 1
      own_tile = ta; own_ka = (int)(u0 - (long long)ta * KT);
      oth_tile = tb; oth_ka = 0; oth_kb = (int)(u1 - (long long)tb * KT);
    }
  }

  const uint32_t wstep32 = (uint32_t)ra.w_step_bytes;

  // ---- K steps ka .. kb-1 of tile `pid` into acc (the ping-pong schedule of gemm_pp_kernel, stage
  // (kt - ka) & 1; every wave passes the same number of barriers).  On return every wave has read
  // its last fragments; the caller must pass a workgroup barrier before LDS is written again.
  auto run_range = [&](int pid, int ka, int kb, floatx16_t (&acc)[TM][TN], float (&rs)[TM], int& m0,
                       int& n0) {
    LZ_FRESH_LANE();
    int tile_m, tile_n;
    workgroup_tile(pid, tiles_m, tiles_n, group_m, tile_m, tile_n);
    m0 = tile_m * BM; n0 = tile_n * BN;
    const int crow = lane >> 3;
    uint32_t koff[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      koff[ks] = (uint32_t)(((ks * 2 + (lane >> 5)) ^ swz64(lane & 31)) * 16);
    const uint32_t a_row = (uint32_t)((wm * TM * 32 + (lane & 31)) * ROW_BYTES);
    const uint32_t w_row = (uint32_t)(BM * ROW_BYTES + (wn * TN * 32 + (lane & 31)) * ROW_BYTES);
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
    // (uniform base + 32-bit per-lane offset: sixteen 64-bit per-lane pointers would not fit the
    // register budget next to the accumulators; the launcher checks that the operands span < 4 GB)
    auto issue_one = [&](int stage, int kt, int q) {
      if (q < A_INSTR)
        g2l16((const char*)A + (uint32_t)(a_off[q] + (uint32_t)kt * (uint32_t)(BK * 2)),
              lds + stage * STAGE_BYTES + (wave * A_INSTR + q) * 1024);
      else
        g2l16((const char*)W + (uint32_t)(w_off[q - A_INSTR] + (uint32_t)kt * wstep32),
              lds + stage * STAGE_BYTES + BM * ROW_BYTES + (wave * W_INSTR + q - A_INSTR) * 1024);
    };
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    bf16x8_t af[2][TM], wf[2][TN];

#define LZ_COMPUTE_COPY_PHASE(stage, ktn)                                                      \
  do {                                                                                         \
    __builtin_amdgcn_s_setprio(1);                                                             \
    _Pragma("unroll") for (int k2 = 0; k2 < 2; ++k2)                                           \
      _Pragma("unroll") for (int i = 0; i < TM; ++i)                                           \
        _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                       \
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[k2][j], af[k2][i], acc[i][j], \
                                                              0, 0, 0);                        \
          if ((k2 * TM + i) * TN + j < NCOPY) issue_one((stage), (ktn), (k2 * TM + i) * TN + j); \
        }                                                                                      \
    _Pragma("unroll") for (int n = 0; n < NCOPY; ++n) {                                        \
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                       \
      __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);                                       \
    }                                                                                          \
    __builtin_amdgcn_sched_group_barrier(0x008, 2 * TM * TN - NCOPY, 0);                       \
    __builtin_amdgcn_s_setprio(0);                                                             \
  } while (0)
#define LZ_MEM_PHASE(st, h)                                                                    \
  do {                                                                                         \
    _Pragma("unroll") for (int k2 = 0; k2 < 2; ++k2) {                                         \
      _Pragma("unroll") for (int i = 0; i < TM; ++i)                                           \
        af[k2][i] = *(const bf16x8_t*)((st) + a_row + i * 32 * ROW_BYTES + koff[2 * (h) + k2]); \
      _Pragma("unroll") for (int j = 0; j < TN; ++j)                                           \
        wf[k2][j] = *(const bf16x8_t*)((st) + w_row + j * 32 * ROW_BYTES + koff[2 * (h) + k2]); \
    }                                                                                          \
  } while (0)
#define LZ_COMPUTE_PHASE()                                                                     \
  do {                                                                                         \
    __builtin_amdgcn_s_setprio(1);                                                             \
    _Pragma("unroll") for (int k2 = 0; k2 < 2; ++k2)                                           \
      _Pragma("unroll") for (int i = 0; i < TM; ++i)                                           \
        _Pragma("unroll") for (int j = 0; j < TN; ++j)                                         \
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[k2][j], af[k2][i], acc[i][j], \
                                                              0, 0, 0);                        \
    __builtin_amdgcn_s_setprio(0);                                                             \
  } while (0)
#define LZ_PHASE_END()                                                                         \
  do {                                                                                         \
    __builtin_amdgcn_sched_barrier(0);                                                         \
    asm volatile("s_barrier" ::: "memory");                                                    \
    __builtin_amdgcn_sched_barrier(0);                                                         \
  } while (0)

#pragma unroll
    for (int q = 0; q < NCOPY; ++q) issue_one(0, ka, q);
    load_row_scales<TM>(rs, ra, M, m0, wm, lane);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (group == 1) LZ_PHASE_END();
    const bool idle_wave = m0 + wm * TM * 32 >= M;
    if (idle_wave) {
      // all of this wave's rows are past M (last tile row): it copies its share of the stages and
      // keeps the barriers, but runs no MFMA (a loop of its own, so that the accumulators of the
      // working waves' loop have one definition)
      for (int kt = ka; kt < kb; ++kt) {
        const int par = (kt - ka) & 1;
        const int k_next = kt + 1 < kb ? kt + 1 : kt;
        LZ_PHASE_END();
#pragma unroll
        for (int q = 0; q < NCOPY; ++q) issue_one(par ^ 1, k_next, q);
        LZ_PHASE_END();
        if (group == 1) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        LZ_PHASE_END();
        if (group == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        LZ_PHASE_END();
      }
    } else
    for (int kt = ka; kt < kb; ++kt) {
      const int par = (kt - ka) & 1;
      const char* cur = lds + par * STAGE_BYTES;
      const int k_next = kt + 1 < kb ? kt + 1 : kt;
      LZ_MEM_PHASE(cur, 0);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      LZ_PHASE_END();
      LZ_COMPUTE_COPY_PHASE(par ^ 1, k_next);
      LZ_PHASE_END();
      LZ_MEM_PHASE(cur, 1);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      if (group == 1) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      LZ_PHASE_END();
      LZ_COMPUTE_PHASE();
      if (group == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      LZ_PHASE_END();
    }
    if (group == 0) LZ_PHASE_END();
#undef LZ_MEM_PHASE
#undef LZ_COMPUTE_PHASE
#undef LZ_COMPUTE_COPY_PHASE
#undef LZ_PHASE_END
  };

  auto finish_tile = [&](floatx16_t (&acc)[TM][TN], const float (&rs)[TM], int m0, int n0) {
    LZ_FRESH_LANE();
    if (EPI == EPI_SWIGLU || !ra.stage_out) {
      gemm_epilogue<TM, TN, EPI>(acc, C, R, M, ldc, m0, n0, wm, wn, lane, ra, rs);
    } else {
      static_assert(BM * ((EPI == EPI_SWIGLU) ? BN / 2 : BN) * 2 <= 2 * STAGE_BYTES, "staged tile must fit the stages");
      staged_tile_out<TM, TN, EPI, BM, BN, NWAVES>(acc, C, R, M, ldc, m0, n0, wm, wn, wave, lane, ra, rs, lds);
    }
    __syncthreads();                                // the next item refills stage 0
  };

  // ---- 1. whole tiles
  for (int r = 0; r < full; ++r) {
    floatx16_t acc[TM][TN];
    float rs[TM];
    int m0, n0;
    run_range(r * G + g, 0, KT, acc, rs, m0, n0);
    finish_tile(acc, rs, m0, n0);
  }

  // ---- 2. the piece of somebody else's tile: partial sums to slot g, then the flag
  if (oth_tile >= 0) {
    floatx16_t acc[TM][TN];
    float rs[TM];
    int m0, n0;
    run_range(sk_pid(oth_tile), oth_ka, oth_kb, acc, rs, m0, n0);
    LZ_FRESH_LANE();
    float4* dst = (float4*)(part + (size_t)g * TILE_FLOATS);
    {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4)
            dst[((wave * (TM * TN) + i * TN + j) * 4 + q4) * 64 + lane] =
                make_float4(acc[i][j][4 * q4], acc[i][j][4 * q4 + 1], acc[i][j][4 * q4 + 2],
                            acc[i][j][4 * q4 + 3]);
        }
      // Every wave's stores have reached the L2 (vmcnt), then the flag goes up.  The reader sits
      // on the same XCD, behind the same L2, so there is nothing to write back or to invalidate
      // (a release fence writes the whole L2 back and an acquire fence empties it for everybody
      // on the XCD, 4-8 us per launch); the flag carries this workgroup's XCC id, and the reader
      // checks that it is its own.
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
    }
    if (threadIdx.x == 0)
      __hip_atomic_store(flags + g, 1u + my_xcc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }

  // ---- 3. the end of the tile this workgroup owns, plus the pieces the others left
  if (own_tile >= 0) {
    floatx16_t acc[TM][TN];
    float rs[TM];
    int m0, n0;
    run_range(sk_pid(own_tile), own_ka, KT, acc, rs, m0, n0);
    if (own_ka > 0) {
      // the tile's other pieces belong to this XCD's workgroups i_first .. gi-1 (ids xcd + 8 i)
      int i_first = gi;
      while (i_first > 0 && ubegin(i_first) > (long long)own_tile * KT) --i_first;
      if (threadIdx.x == 0) {
        unsigned failed = 0;
        for (int ip = i_first; ip < gi; ++ip) {
          if (ubegin(ip + 1) <= ubegin(ip)) continue;         // an empty range wrote nothing
          const int gp = xcd + 8 * ip;
          unsigned spins = 0, seen;
          while ((seen = __hip_atomic_load(flags + gp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) == 0u) {
            __builtin_amdgcn_s_sleep(8);
            if (++spins >= PSK_SPIN_LIMIT) { failed = 1; break; }
          }
          if (seen != 0u && seen != 1u + my_xcc) failed = 1;  // written behind another L2: not visible here
        }
        wait_failed = failed;
        if (failed) atomicAdd(flags + 1023, 1u);              // (the last word counts give-ups)
      }
      __syncthreads();
      LZ_FRESH_LANE();
      if (wait_failed == 0) {
        for (int ip = i_first; ip < gi; ++ip) {               // ascending K order
          if (ubegin(ip + 1) <= ubegin(ip)) continue;
          const float4* src = (const float4*)(part + (size_t)(xcd + 8 * ip) * TILE_FLOATS);
          // four blocks (64 registers, free now that the operand fragments are dead) per round trip
          constexpr int NB = TM * TN, BATCH = 4;
          static_assert(NB % 2 == 0, "blocks are fetched in batches");
#pragma unroll
          for (int b0 = 0; b0 < NB; b0 += BATCH) {
            floatx4_t v[BATCH][4];
            {
#pragma unroll
              for (int u = 0; u < BATCH; ++u)
                if (b0 + u < NB) {
#pragma unroll
                  for (int q4 = 0; q4 < 4; ++q4) {
                    const float4 t = src[((wave * NB + b0 + u) * 4 + q4) * 64 + lane];
                    v[u][q4] = floatx4_t{t.x, t.y, t.z, t.w};
                  }
                }
            }
#pragma unroll
            for (int u = 0; u < BATCH; ++u)
              if (b0 + u < NB) {
                const int i = (b0 + u) / TN, j = (b0 + u) % TN;
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                  acc[i][j][4 * q4] += v[u][q4][0]; acc[i][j][4 * q4 + 1] += v[u][q4][1];
                  acc[i][j][4 * q4 + 2] += v[u][q4][2]; acc[i][j][4 * q4 + 3] += v[u][q4][3];
                }
              }
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
      __syncthreads();
      if (threadIdx.x == 0)
        for (int ip = i_first; ip < gi; ++ip)
          __hip_atomic_store(flags + xcd + 8 * ip, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    finish_tile(acc, rs, m0, n0);
  }
#undef LZ_FRESH_LANE
}

// Fewer tiles than workgroups, the same number on every XCD: a whole number S of workgroups per
// tile makes every range an exact 1/S of ONE tile, so that a workgroup has one piece, S - 1 of S
// leave a partial tile and the owner reads S - 1 (80 tiles: 240 workgroups, three per tile,
// instead of 256 ranges of which most straddle two tiles).  Taken when it keeps 3/4 of the CUs.
static bool psk_pieces_align(int G, int tiles) {
  if (tiles >= G || tiles % 8 != 0) return false;
  const int per_xcd = tiles / 8, S = (G / 8) / per_xcd;
  return S >= 2 && S * per_xcd * 4 >= (G / 8) * 3;
}
static int psk_aligned_grid(int G, int tiles) {
  return psk_pieces_align(G, tiles) ? 8 * ((G / 8) / (tiles / 8)) * (tiles / 8) : G;
}

template <int WM, int WN, int TM, int TN>
static hipError_t launch_psk(const void* A, const void* W, void* C, const void* R, int M, int N,
                             int K, int lda, int ldw, int ldc, int epi, int group_m,
                             const EpiArgs& ra, void* ws, hipStream_t st) {
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  constexpr int LDS_BYTES = 2 * (BM + BN) * ROW_BYTES;
  if (N % BN != 0 || ws == nullptr) return hipErrorInvalidValue;
  // the kernel addresses both operands with 32-bit byte offsets
  if ((unsigned long long)M * lda * 2 >= (1ull << 32) ||
      (unsigned long long)N * (ra.w_blocked ? K : ldw) * 2 >= (1ull << 32))
    return hipErrorInvalidValue;
  const int tiles_m = (M + BM - 1) / BM, tiles_n = N / BN;
  EpiArgs ea = ra;
  ea.w_step_bytes = ra.w_blocked ? (unsigned long long)N * ROW_BYTES : (unsigned long long)ROW_BYTES;
  if (ra.w_blocked) ldw = BK;
  ea.sf_blocks_per_seq = (ea.sf_max_rows + 511) / 512;
  ea.stage_out = (epi == EPI_QKV_ROPE) ? (ra.d_model % BN == 0 && (ra.kv_dim > 0 ? ra.kv_dim : ra.d_model) % BN == 0)
                 : (epi != EPI_SWIGLU && ldc % 8 == 0 && ((uintptr_t)C & 15) == 0);
  const int side = ea.sf_z != nullptr ? ea.sf_blocks_per_seq * ea.sf_batch : 0;
  float* part = (float*)ws;
  unsigned* flags = (unsigned*)((char*)ws + SK_PART_BYTES + SK_TICKET_BYTES);
#define LZ_GEMM(E)                                                                               \
  do {                                                                                           \
    auto kern = gemm_psk_kernel<WM, WN, TM, TN, E>;                                              \
    static int resident = -1;                                                                    \
    if (resident < 0) {                                                                          \
      hipError_t e = hipFuncSetAttribute((const void*)kern,                                      \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES); \
      if (e != hipSuccess) return e;                                                             \
      resident = psk_resident_workgroups(kern, LDS_BYTES);                                       \
    }                                                                                            \
    int G = resident < 256 ? resident : 256;                                                     \
    G &= ~7;                                         /* whole rounds over the 8 XCDs */          \
    G = psk_aligned_grid(G, tiles_m * tiles_n);                                                  \
    if (G < 8 || (size_t)G * BM * BN * sizeof(float) > SK_PART_BYTES || G > PSK_FLAG_WORDS_MAX)  \
      return hipErrorInvalidConfiguration;                                                       \
    hipLaunchKernelGGL(kern, dim3(G + side), dim3(512), LDS_BYTES, st, (const uint16_t*)A,       \
                       (const uint16_t*)W, (uint16_t*)C, (const uint16_t*)R, M, N, K, lda, ldw,  \
                       ldc, tiles_m, tiles_n, group_m, G, part, flags, ea);                      \
  } while (0)
  if (epi == EPI_STORE) LZ_GEMM(EPI_STORE);
  else if (epi == EPI_RESIDUAL) LZ_GEMM(EPI_RESIDUAL);
  else if (epi == EPI_SWIGLU) LZ_GEMM(EPI_SWIGLU);
  else if (epi == EPI_QKV_ROPE) {
    if (ra.head_dim == 64) LZ_GEMM(EPI_QKV_ROPE64);
    else if constexpr (TN >= 4) LZ_GEMM(EPI_QKV_ROPE128);
    else return hipErrorInvalidValue;
  }
  else return hipErrorInvalidValue;
#undef LZ_GEMM
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Stream-K on 128x128 tiles (4 waves of 64x64): for shapes whose tile count does not divide
// over the 256 CUs.  The (tile, K step) pairs are numbered tile-major and cut into G equal
// contiguous ranges, one per persistent workgroup (two fit on a CU).  A workgroup finishes
// every tile it covers completely through the normal epilogue; the at most two tiles it shares
// with a neighbour are written as fp32 partial sums into slot [g][0] (its first tile) or
// [g][1] (its last tile), and a second kernel adds the pieces of each shared tile in workgroup
// order (deterministic) and applies the epilogue.  No workgroup ever waits for another.
// ------------------------------------------------------------------------------------------
constexpr int SK_BM = 128, SK_BN = 128, SK_TILE_ELEMS = SK_BM * SK_BN;

__host__ __device__ inline long long sk_begin(int g, long long U, int G) { return (long long)g * U / G; }

template <int EPI>
__global__ void __launch_bounds__(256)
gemm_sk_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ W,
               uint16_t* __restrict__ C, const uint16_t* __restrict__ R, float* __restrict__ partial,
               int M, int N, int K, int lda, int ldw, int ldc, int tiles_m, int tiles_n, int G,
               unsigned long long* __restrict__ ssq_out, size_t wstep,
               const int32_t* __restrict__ r_rows) {
  constexpr int WM = 2, WN = 2, TM = 2, TN = 2, NWAVES = 4;
  constexpr int BM = SK_BM, BN = SK_BN;
  constexpr int A_INSTR = BM / 8 / NWAVES, W_INSTR = BN / 8 / NWAVES;
  constexpr int STAGE_BYTES = (BM + BN) * ROW_BYTES;
  extern __shared__ __attribute__((aligned(1024))) char lds[];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / WN, wn = wave % WN;
  // consecutive ranges on one XCD (ids are dealt round-robin over the 8 XCDs)
  const int g = (int)(blockIdx.x & 7) * (G >> 3) + (int)(blockIdx.x >> 3);
  const int KT = K / BK;
  const long long U = (long long)tiles_m * tiles_n * KT;
  const long long u0 = sk_begin(g, U, G), u1 = sk_begin(g + 1, U, G);
  if (u0 >= u1) return;
  const int first_tile = (int)(u0 / KT);

  uint32_t koff[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
    koff[ks] = (uint32_t)(((ks * 2 + (lane >> 5)) ^ swz64(lane & 31)) * 16);
  const uint32_t a_row = (uint32_t)((wm * TM * 32 + (lane & 31)) * ROW_BYTES);
  const uint32_t w_row = (uint32_t)(BM * ROW_BYTES + (wn * TN * 32 + (lane & 31)) * ROW_BYTES);
  const int crow = lane >> 3;
  EpiArgs ra{};
  ra.ssq_out = ssq_out;
  ra.r_rows = r_rows;

  long long u = u0;
  while (u < u1) {
    const int tile = (int)(u / KT);
    const int ka = (int)(u - (long long)tile * KT);
    const int kb = (int)min((long long)KT, ka + (u1 - u));
    const int n_it = kb - ka;
    const int tile_m = tile % tiles_m, tile_n = tile / tiles_m;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    uint32_t a_off[A_INSTR], w_off[W_INSTR];
#pragma unroll
    for (int q = 0; q < A_INSTR; ++q) {
      const int tr = (wave * A_INSTR + q) * 8 + crow;
      const int cchunk = (lane & 7) ^ swz64(tr);
      int r = m0 + tr;
      r = r < M ? r : M - 1;
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
    auto issue = [&](int stage, int kt) {
      char* sa = lds + stage * STAGE_BYTES + (wave * A_INSTR) * 1024;
      char* sw = lds + stage * STAGE_BYTES + BM * ROW_BYTES + (wave * W_INSTR) * 1024;
      const char* ga = (const char*)A + (size_t)kt * BK * 2;
      const char* gw = (const char*)W + (size_t)kt * wstep;
#pragma unroll
      for (int q = 0; q < A_INSTR; ++q) g2l16(ga + a_off[q], sa + q * 1024);
#pragma unroll
      for (int q = 0; q < W_INSTR; ++q) g2l16(gw + w_off[q], sw + q * 1024);
    };

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
    issue(0, ka);
    if (n_it > 1) issue(1, ka + 1);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    LZ_LOAD_FRAGS(0, lds, 0);
    for (int it = 0; it < n_it; ++it) {
      const char* cur = lds + (it & 1) * STAGE_BYTES;
      const char* nxt = lds + ((it + 1) & 1) * STAGE_BYTES;
      LZ_LOAD_FRAGS(1, cur, 1);
      LZ_MFMAS(0);
      LZ_LOAD_FRAGS(0, cur, 2);
      LZ_MFMAS(1);
      LZ_LOAD_FRAGS(1, cur, 3);
      LZ_MFMAS(0);
      asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
      __syncthreads();
      if (it + 2 < n_it) issue(it & 1, ka + it + 2);
      if (it + 1 < n_it) LZ_LOAD_FRAGS(0, nxt, 0);
      LZ_MFMAS(1);
    }
#undef LZ_LOAD_FRAGS
#undef LZ_MFMAS
    if (ka == 0 && kb == KT) {
      gemm_epilogue<TM, TN, EPI>(acc, C, R, M, ldc, m0, n0, wm, wn, lane, ra);
    } else {
      // fp32 partial sums of this piece, tile-local row-major [128][128]
      float* dst = partial + ((size_t)g * 2 + (tile == first_tile ? 0 : 1)) * SK_TILE_ELEMS;
      const int tok_l = lane & 31, feat_l = 4 * (lane >> 5);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            float4 v = make_float4(acc[i][j][4 * q4], acc[i][j][4 * q4 + 1], acc[i][j][4 * q4 + 2],
                                   acc[i][j][4 * q4 + 3]);
            *(float4*)(dst + ((wm * TM + i) * 32 + tok_l) * SK_BN + (wn * TN + j) * 32 + 8 * q4 +
                       feat_l) = v;
          }
    }
    u += n_it;
    __syncthreads();            // the next piece refills stage 0: everyone must be done reading
  }
}

// Adds the pieces of every tile that more than one workgroup worked on and applies the
// epilogue.  One workgroup per tile; tiles finished by a single workgroup return at once.
template <int EPI>
__global__ void __launch_bounds__(256)
gemm_sk_fixup_kernel(const float* __restrict__ partial, uint16_t* __restrict__ C,
                     const uint16_t* __restrict__ R, int M, int ldc, int tiles_m, int KT,
                     long long U, int G, unsigned long long* __restrict__ ssq_out,
                     const int32_t* __restrict__ r_rows) {
  const int tile = blockIdx.x;
  const long long ua = (long long)tile * KT, ub = ua + KT - 1;
  // owner(u) = largest g with sk_begin(g) <= u
  int g_first = (int)(ua * G / U), g_last = (int)(ub * G / U);
  while (g_first + 1 < G && sk_begin(g_first + 1, U, G) <= ua) ++g_first;
  while (g_first > 0 && sk_begin(g_first, U, G) > ua) --g_first;
  while (g_last + 1 < G && sk_begin(g_last + 1, U, G) <= ub) ++g_last;
  while (g_last > 0 && sk_begin(g_last, U, G) > ub) --g_last;
  if (g_first == g_last) return;
  // piece pointers are worked out by one thread per batch of 64 (the range arithmetic is
  // 64-bit division); one float4 per thread: blockIdx.y picks an 8-row slab of the tile
  constexpr int MAX_PIECES = 64;
  __shared__ const float* piece[MAX_PIECES];
  __shared__ int n_piece, g_next;
  const int tile_m = tile % tiles_m, tile_n = tile / tiles_m;
  const int m0 = tile_m * SK_BM, n0 = tile_n * SK_BN;
  const int r = blockIdx.y * 8 + (threadIdx.x >> 5), c4 = (threadIdx.x & 31) * 4;
  const int row = m0 + r;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  if (threadIdx.x == 0) g_next = g_first;
  __syncthreads();
  while (true) {
    if (threadIdx.x == 0) {
      int np = 0, g = g_next;
      for (; g <= g_last && np < MAX_PIECES; ++g) {
        const long long b0 = sk_begin(g, U, G), b1 = sk_begin(g + 1, U, G);
        if (b0 >= b1) continue;                                        // empty range
        const int slot = ((int)(b0 / KT) == tile) ? 0 : 1;
        piece[np++] = partial + ((size_t)g * 2 + slot) * SK_TILE_ELEMS;
      }
      n_piece = np;
      g_next = g;
    }
    __syncthreads();
    const int np = n_piece;
    const bool more = g_next <= g_last;
    if (row < M) {
      int p = 0;
      for (; p + 4 <= np; p += 4) {               // four loads in flight, summed in piece order
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = *(const float4*)(piece[p + u] + r * SK_BN + c4);
#pragma unroll
        for (int u = 0; u < 4; ++u) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
      }
      for (; p < np; ++p) {
        const float4 v = *(const float4*)(piece[p] + r * SK_BN + c4);
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
      }
    }
    __syncthreads();
    if (!more) break;
  }
  if (row < M) {
    const size_t off = (size_t)row * ldc + n0 + c4;
    if (EPI == EPI_RESIDUAL) {
      const uint2 r2 = *(const uint2*)(R + (size_t)(r_rows != nullptr ? r_rows[row] : row) * ldc + n0 + c4);
      acc.x += bf16_lo(r2.x); acc.y += bf16_hi(r2.x);
      acc.z += bf16_lo(r2.y); acc.w += bf16_hi(r2.y);
    }
    uint2 w2;
    w2.x = pack_bf16(acc.x, acc.y);
    w2.y = pack_bf16(acc.z, acc.w);
    *(uint2*)(C + off) = w2;
    if (EPI == EPI_RESIDUAL && ssq_out != nullptr) {
      // a row is 32 consecutive lanes (half a wave, all of them past the row < M test together)
      const float a = bf16_lo(w2.x), b = bf16_hi(w2.x), c = bf16_lo(w2.y), e = bf16_hi(w2.y);
      float ss = a * a + b * b + c * c + e * e;
#pragma unroll
      for (int sh = 16; sh >= 1; sh >>= 1) ss += __shfl_xor(ss, sh, 64);
      if ((threadIdx.x & 31) == 0) atomicAdd(ssq_out + row, ssq_to_fixed(ss));
    }
  }
}

static_assert(SK_PART_BYTES == (size_t)SK_GRID * 2 * SK_TILE_ELEMS * sizeof(float), "partial tiles of the 128x128 stream-K form");
size_t gemm_workspace_bytes() { return SK_PART_BYTES + SK_TICKET_BYTES + PSK_FLAG_BYTES; }

static hipError_t launch_sk(const void* A, const void* W, void* C, const void* R, float* partial,
                            int M, int N, int K, int lda, int ldw, int ldc, int epi,
                            unsigned long long* ssq_out, bool w_blocked, const int32_t* r_rows,
                            hipStream_t st) {
  constexpr int LDS_BYTES = 2 * (SK_BM + SK_BN) * ROW_BYTES;
  const size_t wstep = w_blocked ? (size_t)N * ROW_BYTES : (size_t)ROW_BYTES;   // bytes from one K step of a row to the next
  if (w_blocked) ldw = BK;
  const int tiles_m = (M + SK_BM - 1) / SK_BM, tiles_n = N / SK_BN, KT = K / BK;
  const long long U = (long long)tiles_m * tiles_n * KT;
  // Workgroups: as many as are resident at once (two per CU), unless a whole number S of them per
  // tile, with S dividing the K steps, comes close to that: then every range is exactly 1/S of
  // one tile, a workgroup leaves one partial tile instead of two, and the fix-up reads that much
  // less (96 tiles at 355 rows: 384 workgroups, O projection 40.9 -> 36.2 us, down 70.4 -> 61.2).
  int G = SK_GRID;
  for (int S = SK_GRID / (tiles_m * tiles_n); S >= 2; --S)
    if (KT % S == 0) {
      if (tiles_m * tiles_n * S * 10 >= SK_GRID * 7) G = tiles_m * tiles_n * S;
      break;
    }
#define LZ_GEMM(E)                                                                               \
  do {                                                                                           \
    auto kern = gemm_sk_kernel<E>;                                                               \
    static bool attr_set = false;                                                                \
    if (!attr_set) {                                                                             \
      hipError_t e = hipFuncSetAttribute((const void*)kern,                                      \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES); \
      if (e != hipSuccess) return e;                                                             \
      attr_set = true;                                                                           \
    }                                                                                            \
    hipLaunchKernelGGL(kern, dim3(G), dim3(256), LDS_BYTES, st, (const uint16_t*)A,              \
                       (const uint16_t*)W, (uint16_t*)C, (const uint16_t*)R, partial, M, N, K,   \
                       lda, ldw, ldc, tiles_m, tiles_n, G, ssq_out, wstep, r_rows);              \
    hipError_t e = hipGetLastError();                                                            \
    if (e != hipSuccess) return e;                                                               \
    hipLaunchKernelGGL(gemm_sk_fixup_kernel<E>, dim3(tiles_m * tiles_n, 16), dim3(256), 0, st,   \
                       partial, (uint16_t*)C, (const uint16_t*)R, M, ldc, tiles_m, KT, U, G,     \
                       ssq_out, r_rows);                                                         \
  } while (0)
  if (epi == EPI_STORE) LZ_GEMM(EPI_STORE);
  else if (epi == EPI_RESIDUAL) LZ_GEMM(EPI_RESIDUAL);
  else return hipErrorInvalidValue;
#undef LZ_GEMM
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Skinny kernel for M <= 32 token rows (decoding steps): the GEMM is then a stream of the
// weight matrix through the chip and is bound by HBM, not by the matrix pipe, so the job is to
// have every CU pull bytes all the time.  A WAVE owns 128 output features and a range of K and
// runs its own pipeline, with no workgroup barrier in the loop: it copies 128 x 32 slices of W
// (8 KB, whole 64-byte row pieces, global -> LDS) into a private two-slot ring, reads them
// back as MFMA operand fragments, and multiplies them with the 32 token rows (B operand; their
// slice of A rides in the same ring slot, rows past M repeat row M-1; the A matrix is tiny and
// L2-resident).  Everything arrives by global -> LDS copies counted by hand: operands loaded
// into registers across the loop's back edge make the compiler wait for ALL outstanding copies
// before their first use, which serialises the ring (measured: 2 TB/s instead of 5).
// The 4 waves of a workgroup take consecutive K ranges of the same 128 features and add their
// partial sums through LDS in wave order; when K is also split over `ks` workgroups, each leaves
// its partial tile (valid token rows only) in the workspace and takes a ticket from a
// per-column-group counter: whoever draws the last ticket adds all partial tiles in split order
// -- a fixed order, so results do not depend on arrival order -- applies the epilogue and resets
// the counter.  Nobody waits for anybody.  `counters` must be zero on entry.
// ------------------------------------------------------------------------------------------
constexpr int SKN_TN = 4;                         // 32-column blocks per wave: 128 features
constexpr int SKN_TILE = 64 * SKN_TN * 16;        // floats of one partial tile (lane-major)
constexpr int SKN_BK = 32;                        // K elements per pipeline step
constexpr int SKN_WSLOT = SKN_TN * 32 * SKN_BK * 2;       // 8 KB of W
constexpr int SKN_DMA = SKN_WSLOT / 1024;                 // wave-wide copies of W per slot
// a slot = the W slice + the token rows' slice of A (AR = 16 or 32 rows of 64 bytes); 4 waves x 2
// slots = 72 or 80 KB per workgroup.  Two workgroups must fit a CU's 160 KB.
constexpr int skn_slot(int ar) { return SKN_WSLOT + ar * SKN_BK * 2; }
constexpr int skn_lds(int ar) { return 4 * 2 * skn_slot(ar); }
static_assert(3 * SKN_TILE * 4 <= skn_lds(16), "the reduction reuses the rings");

template <int EPI, int AR>
__global__ void __launch_bounds__(256, 2)
gemm_skinny_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ W,
                   uint16_t* __restrict__ C, const uint16_t* __restrict__ R, int M, int K, int lda,
                   int ldw, int ldc, int n_groups, int ks, int steps_per_wave,
                   float* __restrict__ part, unsigned* __restrict__ counters, EpiArgs ra) {
  constexpr int SKN_SLOT = skn_slot(AR);
  constexpr int SKN_OPS = SKN_DMA + AR / 16;       // vector-memory operations per step
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  if ((int)blockIdx.x >= n_groups * ks) {          // side job (see EpiArgs): Eq. 1 scores
    const int sb = (int)blockIdx.x - n_groups * ks;
    score_finish_block<true>(ra.sf_z, ra.sf_stat, ra.sf_s, ra.sf_cu, ra.sf_n_single, ra.sf_heads,
                             ra.sf_z_ld, ra.sf_cu_z, true, sb / ra.sf_blocks_per_seq,
                             (sb % ra.sf_blocks_per_seq) * (int)blockDim.x, (float2*)lds);
    return;
  }
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int hi = lane >> 5, l31 = lane & 31;
  const int cg = blockIdx.x / ks, split = blockIdx.x % ks;
  const int n0 = cg * (SKN_TN * 32);
  const int ksteps = K / SKN_BK;
  const int s_begin = min((split * 4 + wave) * steps_per_wave, ksteps);
  const int n = min(s_begin + steps_per_wave, ksteps) - s_begin;      // steps of this wave

  floatx16_t acc[1][SKN_TN];
#pragma unroll
  for (int j = 0; j < SKN_TN; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[0][j][r] = 0.f;

  // copy plan: instruction t fills rows 16t..16t+15 of the slot, lane p row p/4, stored chunk
  // p%4 = logical chunk (p%4) ^ swz32(row)
  // With ra.w_packed the weight is stored as the sequence of these slot images (see
  // pack_stream_kernel): a step's 8 KB are contiguous in memory and a wave's steps follow each
  // other, so every wave reads one sequential stream instead of 64-byte pieces of 128 rows.
  char* ring = lds + wave * 2 * SKN_SLOT;
  const bool packed = ra.w_packed != 0;
  uint32_t w_off[SKN_DMA];
#pragma unroll
  for (int t = 0; t < SKN_DMA; ++t) {
    const int tr = t * 16 + (lane >> 2);
    w_off[t] = packed ? (uint32_t)(t * 1024 + lane * 16)
                      : (uint32_t)(((size_t)(n0 + tr) * ldw + (((lane & 3) ^ swz32(tr)) * 8)) * 2);
  }
  const size_t w_step = packed ? (size_t)SKN_WSLOT : (size_t)SKN_BK * 2;
  const char* gw = (const char*)W + (packed ? ((size_t)cg * ksteps + s_begin) * SKN_WSLOT
                                            : (size_t)s_begin * SKN_BK * 2);
  auto issue = [&](int slot, int step) {           // step counted from s_begin
#pragma unroll
    for (int t = 0; t < SKN_DMA; ++t)
      g2l16(gw + (size_t)step * w_step + w_off[t], ring + slot * SKN_SLOT + t * 1024);
  };
  // the A slice: one or two more instructions, 16 token rows each
  uint32_t a_off[AR / 16];
#pragma unroll
  for (int u = 0; u < AR / 16; ++u) {
    const int tr = u * 16 + (lane >> 2);
    const int row = tr < M ? tr : M - 1;
    a_off[u] = (uint32_t)(((size_t)row * lda + (((lane & 3) ^ swz32(tr)) * 8)) * 2);
  }
  const char* ga = (const char*)A + (size_t)s_begin * SKN_BK * 2;
  auto issue_all = [&](int slot, int step) {       // step counted from s_begin
    issue(slot, step);
#pragma unroll
    for (int u = 0; u < AR / 16; ++u)
      g2l16(ga + (size_t)step * SKN_BK * 2 + a_off[u], ring + slot * SKN_SLOT + SKN_WSLOT + u * 1024);
  };
  // operand fragments: row j*32 + l31 of the slot (token row l31 of the A part), logical chunk 2q + hi
  // (with 16 token rows in the slot, lanes of tokens 16..31 -- past M -- re-read rows 0..15)
  uint32_t f_off[2], fa_off[2];
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    f_off[q] = (uint32_t)(l31 * 64 + (((q * 2 + hi) ^ swz32(l31)) * 16));
    const int ta = l31 & (AR - 1);
    fa_off[q] = (uint32_t)(ta * 64 + (((q * 2 + hi) ^ swz32(ta)) * 16));
  }

  bf16x8_t af[2], wf[SKN_TN][2];
#define LZ_SKN_STEP(SLOT, NEXT_ISSUED, REFILL)                                                \
  do {                                                                                        \
    __builtin_amdgcn_sched_barrier(0);                                                        \
    if (NEXT_ISSUED) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(SKN_OPS) : "memory");           \
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                                     \
    __builtin_amdgcn_sched_barrier(0);                                                        \
    _Pragma("unroll") for (int q = 0; q < 2; ++q)                                             \
      af[q] = *(const bf16x8_t*)(ring + (SLOT) * SKN_SLOT + SKN_WSLOT + fa_off[q]);           \
    _Pragma("unroll") for (int j = 0; j < SKN_TN; ++j)                                        \
      _Pragma("unroll") for (int q = 0; q < 2; ++q)                                           \
        wf[j][q] = *(const bf16x8_t*)(ring + (SLOT) * SKN_SLOT + j * 32 * 64 + f_off[q]);     \
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                                        \
    __builtin_amdgcn_sched_barrier(0);                                                        \
    if ((REFILL) < n) issue_all(SLOT, REFILL);                                                \
    _Pragma("unroll") for (int q = 0; q < 2; ++q)                                             \
      _Pragma("unroll") for (int j = 0; j < SKN_TN; ++j)                                      \
        acc[0][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j][q], af[q], acc[0][j], 0, 0, 0); \
    __builtin_amdgcn_sched_barrier(0);                                                        \
  } while (0)
  if (n > 0) issue_all(0, 0);
  if (n > 1) issue_all(1, 1);
  for (int i = 0; i < n; i += 2) {
    LZ_SKN_STEP(0, i + 1 < n, i + 2);
    if (i + 1 < n) LZ_SKN_STEP(1, i + 2 < n, i + 3);
  }
#undef LZ_SKN_STEP

  // ---- the four waves' partial sums, added in wave order (the rings are free now)
  __syncthreads();
  float* red = (float*)lds;
  if (wave > 0) {
    float* my = red + (wave - 1) * SKN_TILE;
#pragma unroll
    for (int j = 0; j < SKN_TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) my[(j * 16 + r) * 64 + lane] = acc[0][j][r];
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int w = 0; w < 3; ++w)
#pragma unroll
      for (int j = 0; j < SKN_TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[0][j][r] += red[w * SKN_TILE + (j * 16 + r) * 64 + lane];
  }
  if (ks == 1) {
    if (wave != 0) return;
  } else {
    // ---- K split over workgroups.  Partial tiles go to the workspace as [token][128 features]
    // (valid tokens only); the workgroup that draws the last ticket adds them in split order,
    // all 256 threads at once (one element each per pass, its `ks` loads in flight together:
    // the fix-up costs one trip to memory, not `ks`), and hands the sums back to wave 0.
    __shared__ unsigned last_flag;
    __syncthreads();                                 // (everyone is done reading `red`)
    if (wave == 0) {
      // Agent-scope atomic stores go straight to the level of the memory system that every CU
      // sees; once they have completed (vmcnt) the ticket may be drawn.  A release fence here
      // instead would write back the whole L2's dirty lines, once per workgroup, hundreds of
      // them at the same moment: that alone cost 20-40 us per launch.  The adding threads below
      // read with agent-scope atomic loads, which bypass the non-coherent caches likewise.
      float* slot = part + ((size_t)cg * ks + split) * SKN_TILE;
      if (l31 < M) {
#pragma unroll
        for (int j = 0; j < SKN_TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            __hip_atomic_store(slot + l31 * 128 + j * 32 + 8 * (r / 4) + 4 * hi + (r % 4), acc[0][j][r],
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      if (lane == 0)
        last_flag = __hip_atomic_fetch_add(counters + cg, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                            (unsigned)(ks - 1) ? 1u : 0u;
    }
    __syncthreads();
    if (last_flag == 0) return;
    const float* base = part + (size_t)cg * ks * SKN_TILE;
    for (int e = threadIdx.x; e < M * 128; e += 256) {
      float sum = 0.f;
      for (int sp = 0; sp < ks; sp += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
          v[u] = sp + u < ks ? __hip_atomic_load(base + (size_t)(sp + u) * SKN_TILE + e, __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT)
                             : 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) sum += v[u];
      }
      red[e] = sum;
    }
    if (threadIdx.x == 0) counters[cg] = 0;          // ready for the next launch
    __syncthreads();
    if (wave != 0) return;
    if (l31 < M) {
#pragma unroll
      for (int j = 0; j < SKN_TN; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const float4 v4 = *(const float4*)(red + l31 * 128 + j * 32 + 8 * g + 4 * hi);
          acc[0][j][4 * g] = v4.x; acc[0][j][4 * g + 1] = v4.y; acc[0][j][4 * g + 2] = v4.z; acc[0][j][4 * g + 3] = v4.w;
        }
    }
  }
  gemm_epilogue<1, SKN_TN, EPI>(acc, C, R, M, ldc, 0, n0, 0, 0, lane, ra);
}

constexpr size_t SKN_COUNTER_BYTES = 4096;         // one counter per 128 output features

// W [N][K] -> the skinny kernel's stream layout: for every group of 128 output features and every
// 32-element K step the 8 KB image of that step's LDS slot (row r of the group at 64-byte row r,
// its 16-byte chunk c at position c ^ swz32(r)), groups outermost, steps contiguous.
__global__ void __launch_bounds__(256)
pack_stream_kernel(const uint4* __restrict__ W, int ldw8, int ksteps, size_t n_chunks, uint4* __restrict__ Wp) {
  const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= n_chunks) return;
  const int p = (int)(e & 63), t = (int)((e >> 6) & 7);
  const size_t gs = e >> 9;                          // group * ksteps + step
  const int step = (int)(gs % ksteps);
  const size_t group = gs / ksteps;
  const int tr = t * 16 + (p >> 2);
  const int lc = (p & 3) ^ swz32(tr);
  Wp[e] = W[(group * 128 + tr) * (size_t)ldw8 + step * 4 + lc];
}

// W [N][K] -> K-step-major [K / 64][N][64]: one thread per 16-byte chunk.
__global__ void __launch_bounds__(256)
pack_kblock_kernel(const uint4* __restrict__ W, int ldw8, int N, size_t n_chunks, uint4* __restrict__ Wb) {
  const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= n_chunks) return;
  const int c = (int)(e & 7);
  const size_t rn = e >> 3;                          // kt * N + n
  const size_t kt = rn / N, n = rn % N;
  Wb[e] = W[n * (size_t)ldw8 + kt * 8 + c];
}

hipError_t launch_pack_kblock(const void* W, int N, int K, int ldw, void* Wb, hipStream_t st) {
  if (N <= 0 || K <= 0 || K % BK != 0 || ldw % 8 != 0 || ldw < K || ((uintptr_t)W & 15) != 0 ||
      ((uintptr_t)Wb & 15) != 0)
    return hipErrorInvalidValue;
  const size_t n_chunks = (size_t)N * K / 8;
  hipLaunchKernelGGL(pack_kblock_kernel, dim3((unsigned)((n_chunks + 255) / 256)), dim3(256), 0, st,
                     (const uint4*)W, ldw / 8, N, n_chunks, (uint4*)Wb);
  return hipGetLastError();
}

hipError_t launch_pack_stream(const void* W, int N, int K, int ldw, void* Wp, hipStream_t st) {
  if (N <= 0 || K <= 0 || N % 128 != 0 || K % SKN_BK != 0 || ldw % 8 != 0 || ldw < K ||
      ((uintptr_t)W & 15) != 0 || ((uintptr_t)Wp & 15) != 0)
    return hipErrorInvalidValue;
  const size_t n_chunks = (size_t)N * K / 8;
  hipLaunchKernelGGL(pack_stream_kernel, dim3((unsigned)((n_chunks + 255) / 256)), dim3(256), 0, st,
                     (const uint4*)W, ldw / 8, K / SKN_BK, n_chunks, (uint4*)Wp);
  return hipGetLastError();
}

static hipError_t launch_skinny(const void* A, const void* W, void* C, const void* R, int M, int N,
                                int K, int lda, int ldw, int ldc, int epi, const EpiArgs& ra,
                                void* ws, hipStream_t st) {
  if (M > 32 || N % (SKN_TN * 32) != 0 || (size_t)(N / 128) * 4 > SKN_COUNTER_BYTES)
    return hipErrorInvalidValue;
  if ((lda % 8) != 0 || (ldw % 8) != 0 || ((uintptr_t)A & 15) != 0 || ((uintptr_t)W & 15) != 0)
    return hipErrorInvalidValue;
  const int n_groups = N / (SKN_TN * 32), ksteps = K / SKN_BK;
  // two workgroups per CU are resident (80 KB of LDS each); split K so that the grid is about
  // one such round, with at least four steps per wave
  int ks = (512 + n_groups / 2) / n_groups;
  if (ks < 1) ks = 1;
  const int max_ks = (ksteps + 15) / 16;
  if (ks > max_ks) ks = max_ks;
  const size_t part_bytes = SK_PART_BYTES;
  while (ks > 1 && (size_t)n_groups * ks * SKN_TILE * sizeof(float) > part_bytes) --ks;
  const int steps = (ksteps + 4 * ks - 1) / (4 * ks);
  EpiArgs ea = ra;
  ea.sf_blocks_per_seq = (ea.sf_max_rows + 255) / 256;
  ea.stage_out = 0;
  const int side = ea.sf_z != nullptr ? ea.sf_blocks_per_seq * ea.sf_batch : 0;
  float* part = (float*)ws;
  unsigned* counters = (unsigned*)((char*)ws + part_bytes);
#define LZ_GEMM2(E, AR)                                                                          \
  do {                                                                                           \
    auto kern = gemm_skinny_kernel<E, AR>;                                                       \
    static bool attr_set = false;                                                                \
    if (!attr_set) {                                                                             \
      hipError_t e = hipFuncSetAttribute((const void*)kern,                                      \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, skn_lds(AR)); \
      if (e != hipSuccess) return e;                                                             \
      attr_set = true;                                                                           \
    }                                                                                            \
    hipLaunchKernelGGL(kern, dim3(n_groups * ks + side), dim3(256), skn_lds(AR), st,             \
                       (const uint16_t*)A, (const uint16_t*)W, (uint16_t*)C, (const uint16_t*)R, \
                       M, K, lda, ldw, ldc, n_groups, ks, steps, part, counters, ea);            \
  } while (0)
#define LZ_GEMM(E)                                                                               \
  do {                                                                                           \
    if (M <= 16) LZ_GEMM2(E, 16);                                                                \
    else LZ_GEMM2(E, 32);                                                                        \
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
#undef LZ_GEMM2
  return hipGetLastError();
}

hipError_t launch_gemm_counters_clear(void* sk_ws, hipStream_t st) {
  static_assert(SKN_COUNTER_BYTES == SK_TICKET_BYTES, "ticket area");
  return launch_fill_zero((char*)sk_ws + SK_PART_BYTES, SK_TICKET_BYTES + PSK_FLAG_BYTES, st);
}

__global__ void exchange_check_kernel(const unsigned* __restrict__ give_ups, int32_t* __restrict__ status) {
  if (*give_ups != 0u) atomicOr(status, ST_EXCHANGE);
}

hipError_t launch_gemm_exchange_check(const void* sk_ws, int32_t* status, hipStream_t st) {
  const unsigned* flags = (const unsigned*)((const char*)sk_ws + SK_PART_BYTES + SK_TICKET_BYTES);
  hipLaunchKernelGGL(exchange_check_kernel, dim3(1), dim3(1), 0, st, flags + 1023, status);
  return hipGetLastError();
}

hipError_t launch_gemm(const void* A, const void* W, void* C, const void* R, int M, int N, int K,
                       int lda, int ldw, int ldc, int epilogue, hipStream_t st, const EpiArgs* rope,
                       void* sk_ws, size_t sk_ws_bytes) {
  if (M <= 0) return hipSuccess;
  if (N % 128 != 0 || K % BK != 0) return hipErrorInvalidValue;
  // Bits 8..15 of `epilogue` force a tile configuration and bits 16..21 a band height (tuning
  // hook for measurements); 0 = choose here.
  int cfg = (epilogue >> 8) & 0xff, group_m = (epilogue >> 16) & 0x3f;
  const bool packed_flag = (epilogue & (1 << 30)) != 0, blocked_flag = (epilogue & (1 << 29)) != 0;
  epilogue &= 0xff;
  EpiArgs ra{};
  if (rope != nullptr) ra = *rope;
  if (packed_flag) ra.w_packed = 1;
  if (blocked_flag) ra.w_blocked = 1;
  if (epilogue == EPI_QKV_ROPE) {
    const int kvd = rope != nullptr ? (rope->kv_dim > 0 ? rope->kv_dim : rope->d_model) : 0;
    if (rope == nullptr || (rope->head_dim != 64 && rope->head_dim != 128) ||
        N != rope->d_model + 2 * kvd || rope->d_model % 128 != 0 || kvd % 128 != 0)
      return hipErrorInvalidValue;
  }
  if (group_m == 0) {
    // Band height of the tile walk (tile rows that share a run of W column blocks in an XCD's L2).
    // Measured with cold K-step-major weights, 256x256 tiles, us per launch by band height:
    //   gate/up (86 column blocks)  3376 rows: 2: 536-550, 5: 533, 7: 526-528, 14: 556-561
    //                               2364 rows: 2: 408-410, 5: 402;  1182 rows: 1: 206-209, 2..5: 211-222
    //                               8192 rows: 2: 1269-1277, 3: 1229-1234, 5: 1254, 32: 1527
    //                               4916 rows: 2: 750, 5: 730-734;  1967 rows: 2: 331, 5: 326
    //   QKV (48 column blocks)      3376 rows: 7: 298-303, 14: 308-312;  2364 rows: 5: 206, 10: 207-208
    //                               8192 rows: 3 or 5: 662, 16: 718, 32: 805;  4916 rows: 5: 411-413, 20: 456
    //   O and down projections: within 1 % from 2 to 7 (4 kept).
    //   packed batches              gate/up 41499 rows: 2: 6181, 3: 6353, 5: 6332;  29053 rows: 2: 4276, 3: 4302, 5: 4500
    //                               QKV 41499 rows: 2: 3439, 3: 3302, 5: 3543;  14528 rows: 3: 1184, 5: 1177
    // So: about half the tile rows up to 16 of them, 5 from there, 3 for the tallest (2 for the
    // gate/up shape beyond 40 tile rows); below 8 tile rows the gate/up shape is best walked row by
    // row and the QKV shape column by column.
    const int tm256 = (M + 255) / 256;
    const int tall = tm256 <= 11 ? 5 : tm256 <= 16 ? 7 : tm256 <= 24 ? 5 : 3;
    group_m = epilogue == EPI_QKV_ROPE ? (tm256 < 8 ? tm256 : tall)
              : epilogue == EPI_SWIGLU ? (tm256 < 8 ? 1 : tm256 > 40 ? 2 : tall) : 4;
  }
  if (cfg == 0) {
    // 256x256 tiles on 8 waves in ping-pong phases have the best reuse and keep the matrix pipe
    // fed; when they would leave much of the 256 CUs idle, smaller tiles on 4 waves win.  The
    // rotary epilogue needs a wave to span a whole head (128 columns for head_dim 128).
    // (operands of 4 GB and more: only the 4-wave kernels, which address with 64-bit offsets)
    const bool fits32 = pp_operands_fit_32bit(M, N, K, lda, ldw, ra.w_blocked != 0);
    const long big_tiles = fits32 ? (long)((M + 255) / 256) * (N / 256) : 0;
    // Stream-K pays when the data-parallel grid would leave most CUs idle through a long K
    // loop (measured at M = 355: O projection 46 -> 40 us, down projection 114 -> 70 us); with
    // more tiles the 128x128 partial-sum traffic eats the gain (M = 1182: +-5 %).
    // Fewer 256x256 tiles than CUs, but a whole number (>= 2) of workgroups per tile on every XCD:
    // the persistent stream-K schedule then gives each workgroup one piece of one tile (see
    // psk_aligned_grid).  Measured, cold weights, against the best other form: down projection at
    // 600 / 844 / 1182 / 1400 rows 106 -> 87, 107 -> 100, 153 -> 124, 166 -> 138 us; O projection at
    // 1182 / 1400 rows 68.5 -> 63, 68.7 -> 66.6 (but 50 -> 56 at 600 rows, and at 355 rows the 128x128
    // stream-K form below stays ahead: 62 against 79 us).
    // With the exchange free of cache-wide fences it also pays from 64 tiles on with a short K; there
    // the 192-row tile is taken when its count aligns too and it pads fewer rows (O projection at
    // 600 / 768 / 861 / 1000 rows: 49 -> 46, 56 -> 49, 57 -> 50, 59 -> 57 us; down projection at
    // 861 / 1000 rows, 64 tiles of 256 rows in four pieces each: 111 -> 95, 122 -> 106).
    if ((epilogue == EPI_STORE || epilogue == EPI_RESIDUAL) && ra.psk_ready && sk_ws != nullptr &&
        sk_ws_bytes >= gemm_workspace_bytes() && N % 256 == 0 && fits32) {
      const long t192 = (long)((M + 191) / 192) * (N / 256);
      const long least = K >= 8192 ? 48 : 64;
      const bool ok256 = big_tiles < 128 && big_tiles >= least && psk_pieces_align(256, (int)big_tiles);
      const bool ok192 = K < 8192 && t192 < 128 && t192 >= least && psk_pieces_align(256, (int)t192);
      const long pad256 = (M + 255) / 256 * 256 - M, pad192 = (M + 191) / 192 * 192 - M;
      if (ok192 && (!ok256 || pad192 < pad256)) cfg = 10;
      else if (ok256) cfg = 9;
    }
    if (cfg == 0 && (epilogue == EPI_STORE || epilogue == EPI_RESIDUAL) && sk_ws != nullptr &&
        sk_ws_bytes >= gemm_workspace_bytes()) {
      const long t128 = (long)((M + 127) / 128) * (N / 128);
      if (t128 <= 160 && K / BK >= 32) cfg = 6;
      // with a very long K (the down projection) the split still pays at twice the tiles
      // (M = 1182: 149 us against 155 us for the data-parallel 128x128 tiles)
      else if (t128 <= 320 && K / BK >= 128) cfg = 6;
    }
    // Between 150 and 205 tiles of 256 rows a fifth or more of the CUs would sit idle through
    // the one round; 192-row tiles (wave tile 96x64, no rotary epilogue) make more, shorter
    // tiles of the same work when those still fit one round (measured at M = 2364: O projection
    // 104 -> 90 us, down projection 227 -> 211 us; gate/up at M = 355: 88 -> 77 us).
    const long tiles192 = (long)((M + 191) / 192) * (N / 256);
    // a handful of token rows (decoding): stream the weights, see gemm_skinny_kernel.  Only for
    // callers that keep the ticket counters of the workspace zeroed (ra.skinny).  The partial
    // tiles it exchanges grow with M and with the K split.  Measured against the tile kernels with
    // the weights in each kernel's own order, cold: QKV 28 / 31 / 36 / 46 us at 4 / 8 / 16 / 24 rows
    // against 41; O 15 / 16 / 20 / 23 against 25; gate/up 48 / 51 / 57 / 65 against 59; down (K = 2.7 N,
    // the deepest split) 28 / 32 / 40 / 56 against 35.
    const int skinny_rows = K > 2 * N ? 8 : 16;
    if (ra.skinny && M <= skinny_rows && sk_ws != nullptr && sk_ws_bytes >= gemm_workspace_bytes() &&
        N % 128 == 0 && lda % 8 == 0 && ldw % 8 == 0)
      cfg = 8;
    // Persistent stream-K over the 256x256 tiles when the last data-parallel round would leave
    // much of the chip idle.  The exchange of partial tiles costs about 20 us per launch (256 KB
    // per workgroup out and back through the L2) and the cut tiles share less in the L2, so it pays
    // only from 0.4 of an empty round on (0.3 with the long K of the down projection).  Measured, cold weights:
    // down projection at 4916 / 2364 / 1967 rows 466 -> 401, 228 -> 209, 194 -> 163 us, QKV at 1967
    // rows 206 -> 182 us, O at 4916 rows 183 -> 174 us; gate/up at 3376 rows (4.7 rounds) 517 -> 534:
    // not taken.
    if (cfg == 0 && ra.psk_ready && sk_ws != nullptr && sk_ws_bytes >= gemm_workspace_bytes() &&
        N % 256 == 0 && big_tiles >= 128 && epilogue != EPI_SWIGLU) {     // (gate/up: its own rule below)
      const long rounds = (big_tiles + 255) / 256;
      const double slack = (double)rounds - (double)big_tiles / 256.0;
      if (slack >= (K >= 8192 ? 0.3 : 0.4)) cfg = 9;
    }
    // Gate/up with a last round that is two thirds empty (a single round of 150 - 205 tiles, or
    // 320 - 384 tiles: 1.25 - 1.5 rounds, 64 - 128 remainder tiles of two to four pieces each): the
    // persistent stream-K schedule, on the tile height that fits such a count (both: the one with
    // fewer padding rows).  N = 22016 makes 86 column blocks, so 2 or 4 tile rows qualify.
    // Measured, cold weights, against the best data-parallel form: 300 / 355 rows (2 x 86 tiles of
    // 192 rows) 96 -> 89, 101 -> 93 us; 450 / 512 rows (2 x 86 of 256) 110 -> 108, 115 -> 108;
    // 600 / 700 / 768 rows (4 x 86 of 192) 181 -> 151, 190 -> 165, 198 -> 175; 861 / 1000 rows
    // (4 x 86 of 256) 186 -> 179, 224 -> 196.  Not at 430 tiles (1100 / 1182 rows: 216 -> 222) nor
    // with more rounds (the data-parallel form's tile walk has no counterpart there).
    if (cfg == 0 && epilogue == EPI_SWIGLU && ra.psk_ready && sk_ws != nullptr &&
        sk_ws_bytes >= gemm_workspace_bytes() && N % 256 == 0 && fits32) {
      const long t256 = big_tiles, t192 = (long)((M + 191) / 192) * (N / 256);
      const bool ok256 = (t256 >= 150 && t256 <= 205) || (t256 >= 320 && t256 <= 384);
      const bool ok192 = (t192 >= 150 && t192 <= 205) || (t192 >= 320 && t192 <= 384 && t256 > 256);
      const long pad256 = (M + 255) / 256 * 256 - M, pad192 = (M + 191) / 192 * 192 - M;
      if (ok256 && ok192) cfg = pad192 < pad256 ? 10 : 9;
      else if (ok192) cfg = 10;
      else if (ok256) cfg = 9;
    }
    // The same trade with two rounds of 256-row tiles: 192-row tiles run at about 0.82 of a
    // 256-row tile's time each, so they win when their rounds are fewer by more than that
    // (gate/up at 844 rows: 344 tiles = 2 rounds, 195 us; 430 tiles of 192 rows = 2 shorter
    // rounds, 183 us; at 1182 rows 430 against 602 tiles: 215 against 264 us, not taken).
    const long rounds256 = (big_tiles + 255) / 256, rounds192 = (tiles192 + 255) / 256;
    if (cfg != 0) {}
    else if (N % 256 == 0 && big_tiles >= 150 && epilogue != EPI_QKV_ROPE &&
             (rounds256 == 1 ? (big_tiles <= 205 && tiles192 <= 256)
                             : (rounds256 == 2 && 0.82 * (double)rounds192 < (double)rounds256))) cfg = 7;
    else if (N % 256 == 0 && big_tiles >= 150) cfg = 5;
    // rotary epilogue with 128-wide heads: a wave must hold whole heads (128 columns), so the
    // 128x128 tile is cut into 4 waves of 32x128 (QKV at 229 rows: 46 us against 67 us for the
    // 128x256 tile of 64x128 waves, which makes half as many workgroups; level from 1000 rows on)
    // while they fit one round, the same waves as one 8-wave workgroup per CU on a 128x256 tile with
    // three stages (288 KB of LDS would not hold two of those): QKV at 355 / 394 rows 76 -> 70, 71 -> 67 us
    else if (epilogue == EPI_QKV_ROPE && ra.head_dim == 128)
      cfg = (N % 256 == 0 && (long)((M + 127) / 128) * (N / 256) <= 256) ? 13 : 3;
    else cfg = 2;
    if (cfg == 0) return hipErrorInvalidValue;
  }
  if (ra.w_packed && cfg != 8) return hipErrorInvalidValue;
  if (ra.w_blocked && cfg == 8 && ra.w_stream == nullptr) return hipErrorInvalidValue;
  switch (cfg) {
    case 2:                                             // 128x128, 4 waves of 64x64
            return launch_cfg<2, 2, 2, 2>(A, W, C, R, M, N, K, lda, ldw, ldc, epilogue, group_m, ra, st);
    case 3:                                             // 128x128, 4 waves of 32x128 (whole heads per wave)
            return launch_cfg<4, 1, 1, 4>(A, W, C, R, M, N, K, lda, ldw, ldc, epilogue, group_m, ra, st);
    case 13: if (N % 256) return hipErrorInvalidValue;  // 128x256, 8 waves of 32x128 (whole heads), three stages
            return launch_cfg<4, 2, 1, 4, 3>(A, W, C, R, M, N, K, lda, ldw, ldc, epilogue, group_m, ra, st);
    case 14: if (N % 256) return hipErrorInvalidValue;  // 256x256, 4 waves of 128x128 (one per SIMD)
            return launch_gemm_w4(A, W, C, R, M, N, K, lda, ldw, ldc, epilogue, group_m, ra, st);
    case 4: if (N % 256) return hipErrorInvalidValue;   // 128x256, 4 waves of 64x128
            return launch_cfg<2, 2, 2, 4>(A, W, C, R, M, N, K, lda, ldw, ldc, epilogue, group_m, ra, st);
    case 5:                                             // 256x256, 8 waves of 64x128, ping-pong
    case 7: {                                           // 192x256, 8 waves of 96x64, ping-pong
            EpiArgs rw = ra;                            // (the tile walk's counters live among the flags)
            rw.walk_tickets = (sk_ws != nullptr && sk_ws_bytes >= gemm_workspace_bytes() && ra.psk_ready)
                                  ? (unsigned*)((char*)sk_ws + SK_PART_BYTES + SK_TICKET_BYTES) + WALK_TICKET_WORD
                                  : nullptr;
            return cfg == 5 ? launch_pp<4, 2, 2, 4>(A, W, C, R, M, N, K, lda, ldw, ldc, epilogue, group_m, rw, st)
                            : launch_pp<2, 4, 3, 2>(A, W, C, R, M, N, K, lda, ldw, ldc, epilogue, group_m, rw, st);
    }
    case 9:                                             // 256x256 ping-pong, persistent stream-K
            if (sk_ws == nullptr || sk_ws_bytes < gemm_workspace_bytes() || !ra.psk_ready) return hipErrorInvalidValue;
            return launch_psk<4, 2, 2, 4>(A, W, C, R, M, N, K, lda, ldw, ldc, epilogue, group_m, ra, sk_ws, st);
    case 10:                                            // 192x256 ping-pong, persistent stream-K
            if (sk_ws == nullptr || sk_ws_bytes < gemm_workspace_bytes() || !ra.psk_ready) return hipErrorInvalidValue;
            return launch_psk<2, 4, 3, 2>(A, W, C, R, M, N, K, lda, ldw, ldc, epilogue, group_m, ra, sk_ws, st);
    case 6:                                             // 128x128 stream-K + fix-up
            if (sk_ws == nullptr || sk_ws_bytes < gemm_workspace_bytes()) return hipErrorInvalidValue;
            if (ra.a_rows != nullptr) return hipErrorInvalidValue;   // (no row indirection on its A operand)
            return launch_sk(A, W, C, R, (float*)sk_ws, M, N, K, lda, ldw, ldc, epilogue, ra.ssq_out,
                             ra.w_blocked != 0, ra.r_rows, st);
    case 8:                                             // M <= 32: weight streaming
            if (sk_ws == nullptr || sk_ws_bytes < gemm_workspace_bytes()) return hipErrorInvalidValue;
            if (ra.w_stream != nullptr && !ra.w_packed) {
              ra.w_packed = 1;
              W = ra.w_stream;
            }
            return launch_skinny(A, W, C, R, M, N, K, lda, ldw, ldc, epilogue, ra, sk_ws, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace lz
