// Causal flash-attention prefill over the compacted token set (tokens are stored in ascending
// original position, so causality in the compacted order equals causality in the prompt).
//
// Workgroup = NW waves (4 or 8) = 32*NW queries of one head; each wave owns 32 query rows.
// Keys advance 64 per step; the K tile [64][HD] and the transposed V tile [HD][64] are copied
// global -> LDS by global_load_lds into one of NS stages, NS - 1 steps ahead of their use.
// Both products run on v_mfma_f32_32x32x16_bf16
// in the transposed orientation, so that every lane owns ONE query column:
//   S^T[key][q] = K[key][:] . Q[q][:]        A operand = K rows,   B operand = Q rows
//   O^T[dim][q] = Vt[dim][key] . P^T[key][q]  A operand = Vt rows,  B operand = P^T (registers)
// Row statistics (running max, running sum) are then per-lane scalars, and the fp32 S^T
// accumulator feeds the second product without leaving registers: the MFMA rows of S^T are
// mapped to keys through a fixed permutation (bits 2 and 3 swapped) chosen so that the 8
// accumulator values a lane holds for one 16-key step are exactly the 8 consecutive keys the
// B operand of the second product expects from that lane.
#include <stdlib.h>

#include "common.h"

namespace lz {

constexpr int ATT_BN = 64;    // keys per step

// Two waves share each SIMD (two 4-wave workgroups per CU, or waves w and w+4 of an 8-wave one).
// A step is a matrix phase, a vector phase (softmax), a matrix phase; with equal priorities the
// two waves of a SIMD fall into the same phase and the matrix pipe idles while both do softmax.
// In the 8-wave form the first four waves run at a higher priority: they proceed as if alone
// and the other four fill the pipe they leave idle, which puts the pair in opposite phases.
template <int HD, int NW, int NS>
__global__ void __launch_bounds__(NW * 64, 2)
flash_attn_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                  const uint16_t* __restrict__ vt, uint16_t* __restrict__ o,
                  const int32_t* __restrict__ cu, const int32_t* __restrict__ cu_vt, int n_single,
                  int vt_ld, int n_heads, float scale_log2e, float* __restrict__ z,
                  float2* __restrict__ zstat, int z_ld, int kv_group) {
  constexpr int CHK = HD / 8;                 // 16-byte chunks per K row
  constexpr int KSTEPS = HD / 16;             // k-steps of the first product
  constexpr int HS = HD / 32;                 // 32-row blocks of O^T
  constexpr int K_TILE = ATT_BN * HD * 2;     // bytes
  constexpr int STAGE = 2 * K_TILE;           // K tile + Vt tile
  constexpr int ATT_BM = 32 * NW;             // queries per workgroup
  constexpr int K_INSTR = (ATT_BN * CHK / 64) / NW;  // 1 KB copies per wave for the K tile
  constexpr int V_INSTR = (HD * 8 / 64) / NW;        // ... for the Vt tile
  static_assert(K_INSTR >= 1 && V_INSTR >= 1, "tile copies must cover every wave");
  constexpr int K_ROWS_PER_INSTR = 64 / CHK;
  extern __shared__ __attribute__((aligned(1024))) char lds[];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int head = blockIdx.x, b = blockIdx.z;
  int row0, n;
  seq_range(cu, b, n_single, row0, n);
  const int qblocks = (n + ATT_BM - 1) / ATT_BM;
  if ((int)blockIdx.y >= qblocks) return;
  if (NW == 8) {
    if (wave < 4) __builtin_amdgcn_s_setprio(1);
    else __builtin_amdgcn_s_setprio(0);
  }
  const int qb = qblocks - 1 - blockIdx.y;    // longest blocks first
  const int q0 = qb * ATT_BM;
  const int d = n_heads * HD;
  // grouped-query attention: kv_group query heads read one K,V head; rows of K are kvd wide
  const int kvd = d / kv_group, kvh = head / kv_group;
  const int hi = lane >> 5, l31 = lane & 31;

  // ---- Q fragments (B operand of the first product), straight from global memory
  const int qrow = q0 + wave * 32 + l31;                    // this lane's query
  const int qrow_c = qrow < n ? qrow : n - 1;
  bf16x8_t qf[KSTEPS];
  {
    const uint16_t* qp = q + (size_t)(row0 + qrow_c) * d + head * HD + hi * 8;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) qf[s] = *(const bf16x8_t*)(qp + s * 16);
  }

  // ---- copy plan
  const int ntiles = min((n + ATT_BN - 1) / ATT_BN, (q0 + ATT_BM) / ATT_BN);
  const uint16_t* kbase = k + (size_t)row0 * kvd + kvh * HD;
  const uint16_t* vbase = vt + (size_t)kvh * HD * vt_ld + (cu_vt ? cu_vt[b] : 0);
  auto issue = [&](int stage, int k0) {
    char* sk = lds + stage * STAGE;
    char* sv = sk + K_TILE;
#pragma unroll
    for (int qi = 0; qi < K_INSTR; ++qi) {
      const int slab = wave * K_INSTR + qi;
      const int r = slab * K_ROWS_PER_INSTR + lane / CHK;   // key row inside the tile
      const int c = (lane % CHK) ^ (CHK == 16 ? swz128(r) : swz64(r));
      int key = k0 + r;
      key = key < n ? key : n - 1;
      g2l16(kbase + (size_t)key * kvd + c * 8, sk + slab * 1024);
    }
#pragma unroll
    for (int qi = 0; qi < V_INSTR; ++qi) {
      const int slab = wave * V_INSTR + qi;
      const int r = slab * 8 + (lane >> 3);                 // dim row inside the tile
      const int c = (lane & 7) ^ swz64(r);
      g2l16(vbase + (size_t)r * vt_ld + k0 + c * 8, sv + slab * 1024);
    }
  };

  // ---- operand addresses
  const int kperm = (l31 & 0x13) | ((l31 & 4) << 1) | ((l31 & 8) >> 1);   // swap bits 2 and 3
  uint32_t k_addr[2];                       // per 32-key block; chunk term added per k-step
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) k_addr[sub] = (uint32_t)((sub * 32 + kperm) * HD * 2);
  const int kx = CHK == 16 ? swz128(kperm) : swz64(kperm);
  const uint32_t v_addr = (uint32_t)(K_TILE + l31 * 128);
  const int vx = swz64(l31);

  floatx16_t oacc[HS];
#pragma unroll
  for (int h = 0; h < HS; ++h)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[h][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  const int q_lo = q0 + wave * 32, q_hi = q_lo + 31;     // this wave's query range
  const bool score_wave = z != nullptr && q_lo <= n - 1 && n - 1 <= q_hi;   // owns the last query

  // One 64-key step has five parts, with the LDS reads of each part issued under the MFMAs of
  // the part before (two buffers fa/fb of KSTEPS fragments, reads and MFMAs interleaved one
  // for one by scheduling fences; left alone the compiler pairs every MFMA with its own read
  // and waits for it):
  //   1  S^T block 0 from fa (read under part 5 of the step before)   reads K block 1 -> fb
  //   2  S^T block 1 from fb                                          reads Vt half 0 -> fa
  //   3  softmax of the 64 keys (vector unit; the other wave on the SIMD fills the matrix pipe)
  //      -- wait for the copies of step it+1, workgroup barrier, issue the copies of step it+NS-1
  //   4  O^T half 0 from fa                                           reads Vt half 1 -> fb
  //   5  O^T half 1 from fb                                           reads K block 0 of it+1 -> fa
  // The barrier sits after the softmax so that the reads of the next step's K rows can start
  // under part 5: past it every wave's share of step it+1 has landed, and every wave has
  // finished step it-1, whose stage the new copies overwrite.  A bare s_barrier, not
  // __syncthreads, which would make the compiler wait for every outstanding copy.
  //
  // The causal mask costs a compare and a select per element, so only steps that straddle the
  // diagonal of this wave's queries branch into it.  The running maximum is raised only when a
  // step's maximum exceeds it by more than 2^8 (base-2 domain): softmax is invariant to the
  // shift, p stays below 2^8 (fp32 sums and bf16 P keep their relative precision), and the
  // rescale of the O^T accumulators leaves the common path.  The 1/sqrt(hd) * log2(e) scale
  // rides in the fused multiply-add that forms the exponent.
#define LZ_ATT_INTERLEAVE()                                  \
  _Pragma("unroll") for (int g = 0; g < KSTEPS; ++g) {        \
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);        \
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);        \
  }
  constexpr int PER_STEP = K_INSTR + V_INSTR;            // copies one wave issues per step
  constexpr int SCORE_STORES = 8;                        // logit stores per step (score wave)
  static_assert((NS - 3) * (PER_STEP + SCORE_STORES) + SCORE_STORES < 64, "vmcnt is 6 bits");
  static_assert(NS >= 3, "the copies of step it+1 must be issued before step it");
  bf16x8_t fa[KSTEPS], fb[KSTEPS];
  auto kread = [&](const char* st, int sub, int s) {
    return *(const bf16x8_t*)(st + k_addr[sub] + (((s * 2 + hi) ^ kx) * 16));
  };
  auto vread = [&](const char* st, int i) {          // i = 4 * h + 2 * sub + t
    const int chunk = ((i >> 1) & 1) * 4 + (i & 1) * 2 + hi;
    return *(const bf16x8_t*)(st + v_addr + (i >> 2) * 32 * 128 + ((chunk ^ vx) * 16));
  };

#pragma unroll
  for (int t = 0; t < NS - 1; ++t)
    if (t < ntiles) issue(t, t * ATT_BN);
  if (ntiles >= NS - 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 2) * PER_STEP) : "memory");
  else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("s_barrier" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int s = 0; s < KSTEPS; ++s) fa[s] = kread(lds, 0, s);

  int stage_c = 0, stage_i = NS - 1;                     // stage computed / stage copied into
  for (int it = 0; it < ntiles; ++it) {
    const int k0 = it * ATT_BN;
    const char* st = lds + stage_c * STAGE;
    const int stage_n = stage_c + 1 == NS ? 0 : stage_c + 1;
    const bool active = k0 <= q_hi && q_lo < n;   // else every key is in the future, or every query past the end
    bf16x8_t pf[2][2];
    if (active) {
      floatx16_t sacc[2];
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[sub][r] = 0.f;
      // part 1
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s) fb[s] = kread(st, 1, s);
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s)
        sacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[s], qf[s], sacc[0], 0, 0, 0);
      LZ_ATT_INTERLEAVE();
      __builtin_amdgcn_sched_barrier(0);
      // part 2
#pragma unroll
      for (int i = 0; i < KSTEPS; ++i) fa[i] = vread(st, i);
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s)
        sacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[s], qf[s], sacc[1], 0, 0, 0);
      LZ_ATT_INTERLEAVE();
      __builtin_amdgcn_sched_barrier(0);
      // part 3.  Register r of block sub is key k0 + 32*sub + 16*(r/8) + 8*hi + r%8.
      if ((k0 + ATT_BN - 1) > q_lo) {
        asm volatile("; causal mask" ::: "memory");   // keeps this a real branch
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = k0 + 32 * sub + 16 * (r / 8) + 8 * hi + (r % 8);
            if (key > qrow) sacc[sub][r] = -INFINITY;
          }
      }
      // Eq. 1 rides along: the lanes that own the sequence's last query already hold its
      // logits against every key, so they leave them (base-2 domain) for the score kernel.
      if (score_wave) {
        asm volatile("; last-query logits" ::: "memory");
        if (qrow == n - 1) {
          // 16-byte stores into the padded layout of the Vt buffer (sequences start at multiples
          // of 64, so the keys past the sequence's end that a step covers still fall inside)
          float* zr = z + (size_t)head * z_ld + (cu_vt ? cu_vt[b] : 0) + k0 + 8 * hi;
#pragma unroll
          for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              float4 v4;
              v4.x = sacc[sub][4 * g] * scale_log2e;     v4.y = sacc[sub][4 * g + 1] * scale_log2e;
              v4.z = sacc[sub][4 * g + 2] * scale_log2e; v4.w = sacc[sub][4 * g + 3] * scale_log2e;
              *(float4*)(zr + 32 * sub + 16 * (g >> 1) + 4 * (g & 1)) = v4;
            }
        }
      }
      float mraw = -INFINITY;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) mraw = fmaxf(mraw, sacc[sub][r]);
      float mloc = mraw * scale_log2e;
      mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
      if (__builtin_amdgcn_ballot_w64(mloc > m_run + 8.0f) != 0) {
        // The empty asm keeps this a real branch: the compiler would otherwise run the rescale
        // every step under a select.
        const float m_new = fmaxf(m_run, mloc);
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        l_run *= alpha;
        asm volatile("; raise the running maximum" ::: "memory");
#pragma unroll
        for (int h = 0; h < HS; ++h) oacc[h] *= alpha;
      }
      const float neg_m = -m_run;
      float psum = 0.f;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          float p[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            p[j] = __builtin_amdgcn_exp2f(fmaf(sacc[sub][8 * t + j], scale_log2e, neg_m));
            psum += p[j];
          }
          uint4 packed = pack8(p);
          pf[sub][t] = *reinterpret_cast<bf16x8_t*>(&packed);
        }
      l_run += psum;
    }
    // the copies of step it+1 have landed; nobody reads the stage of step it-1 any more
    __builtin_amdgcn_sched_barrier(0);
    // (the wave that also stores the last query's logits has SCORE_STORES more operations in
    // flight per step; they complete in issue order with the copies)
    if (it + NS - 1 > ntiles) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else if (score_wave)
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 3) * (PER_STEP + SCORE_STORES) + SCORE_STORES) : "memory");
    else asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 3) * PER_STEP) : "memory");
    asm volatile("s_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    if (it + NS - 1 < ntiles) issue(stage_i, k0 + (NS - 1) * ATT_BN);
    if (active) {
      // part 4
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < KSTEPS; ++i) fb[i] = vread(st, KSTEPS + i);
#pragma unroll
      for (int i = 0; i < KSTEPS; ++i)
        oacc[i >> 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], pf[(i >> 1) & 1][i & 1],
                                                               oacc[i >> 2], 0, 0, 0);
      LZ_ATT_INTERLEAVE();
      __builtin_amdgcn_sched_barrier(0);
      // part 5 (the reads past the last step fetch a stage nobody uses; they stay inside LDS)
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s) fa[s] = kread(lds + stage_n * STAGE, 0, s);
#pragma unroll
      for (int i = 0; i < KSTEPS; ++i)
        oacc[HS / 2 + (i >> 2)] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            fb[i], pf[(i >> 1) & 1][i & 1], oacc[HS / 2 + (i >> 2)], 0, 0, 0);
      LZ_ATT_INTERLEAVE();
      __builtin_amdgcn_sched_barrier(0);
    }
    stage_c = stage_n;
    stage_i = stage_i + 1 == NS ? 0 : stage_i + 1;
  }
#undef LZ_ATT_INTERLEAVE

  // ---- normalise and store.  Register r of block h is dim 32h + 8*(r/4) + 4*hi + r%4.
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.0f / l_tot;
  if (score_wave && qrow == n - 1 && hi == 0)            // reference point and 1 / sum for Eq. 1
    zstat[(size_t)b * n_heads + head] = make_float2(m_run, inv);
  if (qrow < n) {
    uint16_t* op = o + (size_t)(row0 + qrow) * d + head * HD + 4 * hi;
#pragma unroll
    for (int h = 0; h < HS; ++h)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 w2;
        w2.x = pack_bf16(oacc[h][4 * g] * inv, oacc[h][4 * g + 1] * inv);
        w2.y = pack_bf16(oacc[h][4 * g + 2] * inv, oacc[h][4 * g + 3] * inv);
        *(uint2*)(op + h * 32 + 8 * g) = w2;
      }
  }
}

// ------------------------------------------------------------------------------------------
// Ping-pong form for long sequences (8 waves = 256 queries of one head per workgroup, NS stages).
// The flash_attn_kernel above keeps all eight waves in step (one barrier per 64-key step, after
// the softmax), so the two waves of a SIMD do their matrix work at the same time and their
// vector work at the same time, and the matrix pipe idles through every softmax.  Measured on
// this part, matrix and vector instructions of two waves on one SIMD DO run side by side (32
// MFMAs against 32 fma + exp2 + add groups: 0.60 us together, 0.56 us for the MFMAs alone), so
// here the two waves of a SIMD (w and w + 4) run half a step apart, as in the GEMM's ping-pong
// schedule: a wave alternates a MATRIX half step  M(i) = [O^T += Vt(i-1) P^T(i-1)] [S^T(i) = K(i) Q^T]
// (32 MFMAs back to back, the LDS reads of the next operands in their shadow) and a VECTOR half
// step  V(i) = softmax of step i's 64 keys (mask, running maximum, exp2, bf16 P), and while one
// wave of the pair is in M the other is in V.  A bare s_barrier closes every phase:
//   phase:       0      1      2      3      4    ...
//   waves 0-3:  M(0)   V(0)   M(1)   V(1)   M(2)  ...
//   waves 4-7:   -     M(0)   V(0)   M(1)   V(1)  ...
// Tile t (K rows and Vt columns of keys 64t .. 64t+63) is copied into stage t mod NS by all
// waves at the start of phase 2(t - NS + 1) + 2, when nobody reads tile t - NS any more (its last
// use is M(t - NS + 1) of waves 4-7 in phase 2(t - NS + 1) + 1); every wave waits for its share of
// tile i + 1 before the barrier that ends phase 2i + 1, so M(i + 1) finds it complete.
// ------------------------------------------------------------------------------------------
template <int HD, int NS>
__global__ void __launch_bounds__(512)
flash_attn_pp_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                     const uint16_t* __restrict__ vt, uint16_t* __restrict__ o,
                     const int32_t* __restrict__ cu, const int32_t* __restrict__ cu_vt, int n_single,
                     int vt_ld, int n_heads, float scale_log2e, float* __restrict__ z,
                     float2* __restrict__ zstat, int z_ld, int kv_group) {
  constexpr int NW = 8;
  constexpr int CHK = HD / 8;
  constexpr int KSTEPS = HD / 16;
  constexpr int HS = HD / 32;
  constexpr int K_TILE = ATT_BN * HD * 2;
  constexpr int STAGE = 2 * K_TILE;
  constexpr int ATT_BM = 32 * NW;
  constexpr int K_INSTR = (ATT_BN * CHK / 64) / NW;
  constexpr int V_INSTR = (HD * 8 / 64) / NW;
  static_assert(K_INSTR >= 1 && V_INSTR >= 1, "tile copies must cover every wave");
  static_assert(NS >= 4, "a tile is copied two steps before its first use");
  constexpr int K_ROWS_PER_INSTR = 64 / CHK;
  extern __shared__ __attribute__((aligned(1024))) char lds[];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int group = wave >> 2;
  const int head = blockIdx.x, b = blockIdx.z;
  int row0, n;
  seq_range(cu, b, n_single, row0, n);
  const int qblocks = (n + ATT_BM - 1) / ATT_BM;
  if ((int)blockIdx.y >= qblocks) return;
  const int qb = qblocks - 1 - blockIdx.y;    // longest blocks first
  const int q0 = qb * ATT_BM;
  const int d = n_heads * HD;
  const int kvd = d / kv_group, kvh = head / kv_group;
  const int hi = lane >> 5, l31 = lane & 31;

  const int qrow = q0 + wave * 32 + l31;
  const int qrow_c = qrow < n ? qrow : n - 1;
  bf16x8_t qf[KSTEPS];
  {
    const uint16_t* qp = q + (size_t)(row0 + qrow_c) * d + head * HD + hi * 8;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) qf[s] = *(const bf16x8_t*)(qp + s * 16);
  }

  const int ntiles = min((n + ATT_BN - 1) / ATT_BN, (q0 + ATT_BM) / ATT_BN);
  const uint16_t* kbase = k + (size_t)row0 * kvd + kvh * HD;
  const uint16_t* vbase = vt + (size_t)kvh * HD * vt_ld + (cu_vt ? cu_vt[b] : 0);
  // Lane offsets of this wave's copies inside a tile (bytes, 32 bits): a whole tile is then copied
  // from a uniform base that advances by scalar arithmetic, with no vector work per copy.  Only the
  // sequence's last, partial tile clamps its key rows lane by lane.
  uint32_t k_off[K_INSTR], v_off[V_INSTR];
#pragma unroll
  for (int qi = 0; qi < K_INSTR; ++qi) {
    const int slab = wave * K_INSTR + qi;
    const int r = slab * K_ROWS_PER_INSTR + lane / CHK;
    const int c = (lane % CHK) ^ (CHK == 16 ? swz128(r) : swz64(r));
    k_off[qi] = (uint32_t)(((size_t)r * kvd + c * 8) * 2);
  }
#pragma unroll
  for (int qi = 0; qi < V_INSTR; ++qi) {
    const int slab = wave * V_INSTR + qi;
    const int r = slab * 8 + (lane >> 3);
    const int c = (lane & 7) ^ swz64(r);
    v_off[qi] = (uint32_t)(((size_t)r * vt_ld + c * 8) * 2);
  }
  auto issue = [&](int t) {                    // tile t into stage t mod NS
    char* sk = lds + (t % NS) * STAGE;
    char* sv = sk + K_TILE;
    const int k0 = t * ATT_BN;
    if (k0 + ATT_BN <= n) {
      const char* kt = (const char*)(kbase + (size_t)k0 * kvd);
#pragma unroll
      for (int qi = 0; qi < K_INSTR; ++qi) g2l16(kt + k_off[qi], sk + (wave * K_INSTR + qi) * 1024);
    } else {
#pragma unroll
      for (int qi = 0; qi < K_INSTR; ++qi) {
        const int slab = wave * K_INSTR + qi;
        const int r = slab * K_ROWS_PER_INSTR + lane / CHK;
        const int c = (lane % CHK) ^ (CHK == 16 ? swz128(r) : swz64(r));
        int key = k0 + r;
        key = key < n ? key : n - 1;
        g2l16(kbase + (size_t)key * kvd + c * 8, sk + slab * 1024);
      }
    }
    const char* vt0 = (const char*)(vbase + k0);
#pragma unroll
    for (int qi = 0; qi < V_INSTR; ++qi) g2l16(vt0 + v_off[qi], sv + (wave * V_INSTR + qi) * 1024);
  };

  const int kperm = (l31 & 0x13) | ((l31 & 4) << 1) | ((l31 & 8) >> 1);   // swap bits 2 and 3
  uint32_t k_addr[2];
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) k_addr[sub] = (uint32_t)((sub * 32 + kperm) * HD * 2);
  const int kx = CHK == 16 ? swz128(kperm) : swz64(kperm);
  const uint32_t v_addr = (uint32_t)(K_TILE + l31 * 128);
  const int vx = swz64(l31);

  floatx16_t oacc[HS];
#pragma unroll
  for (int h = 0; h < HS; ++h)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[h][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  const int q_lo = q0 + wave * 32, q_hi = q_lo + 31;
  const bool score_wave = z != nullptr && q_lo <= n - 1 && n - 1 <= q_hi;
  // steps in which this wave has anything to do: keys 64 i .. up to its last query
  const int n_act = q_lo < n ? min(ntiles, q_hi / ATT_BN + 1) : 0;

#define LZ_ATT_INTERLEAVE()                                  \
  _Pragma("unroll") for (int g = 0; g < KSTEPS; ++g) {        \
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);        \
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);        \
  }
#define LZ_PHASE_END()                                       \
  do {                                                       \
    __builtin_amdgcn_sched_barrier(0);                       \
    asm volatile("s_barrier" ::: "memory");                  \
    __builtin_amdgcn_sched_barrier(0);                       \
  } while (0)
  constexpr int PER_STEP = K_INSTR + V_INSTR;
  constexpr int SCORE_STORES = 8;
  static_assert((NS - 3) * PER_STEP + SCORE_STORES < 64, "vmcnt is 6 bits");
  // ---- operand fragments.  One product is NF = 2 * KSTEPS MFMAs, each with its own 16-byte-per-lane
  // fragment from LDS, and the fragments live in ONE ring of NF registers: right after MFMA u has
  // taken slot u, the read of the fragment that the MFMA NF places later needs goes into the same
  // slot -- the first product's MFMAs fetch the Vt fragments of the second product, the second
  // product's the K fragments of the next step's first product.  Every read thus has NF MFMAs
  // (512 cycles at head_dim 128) to come back, and since LDS returns in order the wait in front of
  // an MFMA is always "all but the NF - 1 youngest reads": s_waitcnt lgkmcnt(NF - 1).  The reads
  // and waits are written as asm so that they are exactly these: left to the compiler, a group of
  // reads was followed by a wait for ALL of them (the youngest issued 32 cycles earlier), and a
  // branch in between made it wait for everything outstanding.
  constexpr int NF = 2 * KSTEPS;
  static_assert(NF - 1 <= 15, "lgkmcnt has 4 bits");
  bf16x8_t fr[NF];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
  // lane parts of the fragment addresses (K: k-step s of key block `sub`; Vt: see vread)
  uint32_t k_lane[KSTEPS], v_lane[4];
#pragma unroll
  for (int sidx = 0; sidx < KSTEPS; ++sidx) k_lane[sidx] = lds0 + k_addr[0] + (uint32_t)((((sidx * 2 + hi) ^ kx)) * 16);
#pragma unroll
  for (int c4 = 0; c4 < 4; ++c4) {                     // c4 = 2 * sub + t of vread's index
    const int chunk = ((c4 >> 1) & 1) * 4 + (c4 & 1) * 2 + hi;
    v_lane[c4] = lds0 + v_addr + (uint32_t)((chunk ^ vx) * 16);
  }
#define LZ_LDS_READ(dst, addr, OFF) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF))
#define LZ_FRAG_READY(f) asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(f) : "n"(NF - 1))
  // slot u of the first product: key block u & 1, k-step (u >> 1) % (KSTEPS / 2) + (KSTEPS / 2) * (u / KSTEPS)
  constexpr int HK = KSTEPS / 2;
  auto k_step_of = [](int u) { return ((u % KSTEPS) >> 1) + HK * (u / KSTEPS); };
  // slot u of the second product: Vt operand pv(u) = 4 h + 2 sub + t, alternating output blocks
  auto pv_op = [](int u) { return (u & 1) * (KSTEPS / 2) + (u >> 1); };   // 0,4,1,5,...
  auto v_index_of = [&](int u) { return (u / KSTEPS) * KSTEPS + pv_op(u % KSTEPS); };
  auto read_k_slot = [&](uint32_t stage_off, int u) {  // K fragment of slot u from the stage at stage_off
    const uint32_t addr = k_lane[k_step_of(u)] + stage_off;
    if (u & 1) LZ_LDS_READ(fr[u], addr, 32 * HD * 2);
    else LZ_LDS_READ(fr[u], addr, 0);
  };
  auto read_v_slot = [&](uint32_t stage_off, int u) {  // Vt fragment of slot u
    const int vi = v_index_of(u);
    const uint32_t addr = v_lane[vi & 3] + stage_off;
    switch (vi >> 2) {
      case 0: LZ_LDS_READ(fr[u], addr, 0); break;
      case 1: LZ_LDS_READ(fr[u], addr, 32 * 128); break;
      case 2: LZ_LDS_READ(fr[u], addr, 2 * 32 * 128); break;
      default: LZ_LDS_READ(fr[u], addr, 3 * 32 * 128); break;
    }
  };

  floatx16_t sacc[2];
  bf16x8_t pf[2][2];

  // first product of step i (the ring holds tile i's K fragments; leaves tile i's Vt fragments in it)
  auto first_product = [&](int i) {
    const uint32_t st = (uint32_t)((i % NS) * STAGE);
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[sub][r] = 0.f;
#pragma unroll
    for (int u = 0; u < NF; ++u) {
      LZ_FRAG_READY(fr[u]);
      sacc[u & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[u], qf[k_step_of(u)], sacc[u & 1], 0, 0, 0);
      read_v_slot(st, u);
    }
  };
  // second product of step i (the ring holds tile i's Vt fragments; leaves the K fragments of the
  // stage of tile i + 1 in it -- stale bytes of a valid stage after the last tile, never used)
  auto second_product = [&](int i) {
    const uint32_t st_next = (uint32_t)(((i + 1) % NS) * STAGE);
#pragma unroll
    for (int u = 0; u < NF; ++u) {
      const int op = pv_op(u % KSTEPS), ob = (u / KSTEPS) * (HS / 2) + (op >> 2);
      LZ_FRAG_READY(fr[u]);
      oacc[ob] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[u], pf[(op >> 1) & 1][op & 1], oacc[ob], 0, 0, 0);
      read_k_slot(st_next, u);
    }
  };

  // ---- vector half step i: softmax of the 64 keys of step i (sacc -> pf, running statistics).
  // Register r of block sub is key k0 + 32*sub + 16*(r/8) + 8*hi + r%8.
  auto vector_half = [&](int i) {
    if (i >= n_act) return;
    const int k0 = i * ATT_BN;
    if ((k0 + ATT_BN - 1) > q_lo) {
      asm volatile("; causal mask" ::: "memory");   // keeps this a real branch
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + 32 * sub + 16 * (r / 8) + 8 * hi + (r % 8);
          if (key > qrow) sacc[sub][r] = -INFINITY;
        }
    }
    if (score_wave) {
      asm volatile("; last-query logits" ::: "memory");
      if (qrow == n - 1) {
        float* zr = z + (size_t)head * z_ld + (cu_vt ? cu_vt[b] : 0) + k0 + 8 * hi;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            float4 v4;
            v4.x = sacc[sub][4 * g] * scale_log2e;     v4.y = sacc[sub][4 * g + 1] * scale_log2e;
            v4.z = sacc[sub][4 * g + 2] * scale_log2e; v4.w = sacc[sub][4 * g + 3] * scale_log2e;
            *(float4*)(zr + 32 * sub + 16 * (g >> 1) + 4 * (g & 1)) = v4;
          }
      }
    }
    // (two independent chains; the two lanes of a query, l and l ^ 32, exchange their maxima with
    // v_permlane32_swap: __shfl_xor would be an LDS round trip in the middle of the half step)
    float mraw0 = -INFINITY, mraw1 = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      mraw0 = fmaxf(mraw0, sacc[0][r]);
      mraw1 = fmaxf(mraw1, sacc[1][r]);
    }
    float mloc = fmaxf(mraw0, mraw1) * scale_log2e;
    {
      const unsigned mbits = __float_as_uint(mloc);
      const auto sw = __builtin_amdgcn_permlane32_swap(mbits, mbits, false, false);
      mloc = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
    }
    if (__builtin_amdgcn_ballot_w64(mloc > m_run + 8.0f) != 0) {
      const float m_new = fmaxf(m_run, mloc);
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      m_run = m_new;
      l_run *= alpha;
      asm volatile("; raise the running maximum" ::: "memory");
#pragma unroll
      for (int h = 0; h < HS; ++h) oacc[h] *= alpha;
    }
    const float neg_m = -m_run;
    float psum[4] = {0.f, 0.f, 0.f, 0.f};          // (four chains; added in a fixed order)
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        float p[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          p[j] = __builtin_amdgcn_exp2f(fmaf(sacc[sub][8 * t + j], scale_log2e, neg_m));
          psum[2 * sub + t] += p[j];
        }
        uint4 packed = pack8(p);
        pf[sub][t] = *reinterpret_cast<bf16x8_t*>(&packed);
      }
    l_run += (psum[0] + psum[1]) + (psum[2] + psum[3]);
  };
  // own copies of tile t have landed (tile t+1 may still be in flight; the wave that stores the
  // last query's logits has up to SCORE_STORES more operations behind the copies)
  auto wait_tile = [&](int t, bool stores_behind = true) {
    if (t >= ntiles) return;
    if (t + NS - 3 < ntiles) {                       // tiles t+1 .. t+NS-3 are in flight behind it
      if (score_wave && stores_behind) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 3) * PER_STEP + SCORE_STORES) : "memory");
      else asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 3) * PER_STEP) : "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
  };

  // ---- prologue: tiles 0 .. NS-2 on their way, tile 0 landed
#pragma unroll
  for (int t = 0; t < NS - 1; ++t)
    if (t < ntiles) issue(t);
  if (ntiles >= NS - 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 2) * PER_STEP) : "memory");
  else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  LZ_PHASE_END();
#pragma unroll
  for (int u = 0; u < NF; ++u) read_k_slot(0u, u);   // tile 0's K fragments

  // One instruction stream for both halves of the workgroup; waves 4-7 run it one phase later.
  //   waves 0-3: M(0) in phase 0, then V(i) in phase 2i+1 and M(i+1) in phase 2i+2
  //   waves 4-7: M(0) in phase 1, then V(i) in phase 2i+2 and M(i+1) in phase 2i+3
  // where M(0) is the first product of step 0 and M(i+1) the second product of step i followed by the
  // first product of step i+1.  Tile i+NS-1 is issued at the start of phase 2i+2; tile i+1 is waited
  // for before the barrier that ends phase 2i+1.
  if (group == 1) LZ_PHASE_END();
  if (n_act > 0) {
    __builtin_amdgcn_s_setprio(1);
    first_product(0);
    __builtin_amdgcn_s_setprio(0);
  }
  if (group == 1) wait_tile(1, false);            // (no logit stores issued yet)
  LZ_PHASE_END();
  for (int i = 0; i < ntiles; ++i) {
    if (group == 1 && i + NS - 1 < ntiles) issue(i + NS - 1);
    vector_half(i);
    __builtin_amdgcn_sched_barrier(0);
    if (group == 0) wait_tile(i + 1);
    LZ_PHASE_END();
    if (group == 0 && i + NS - 1 < ntiles) issue(i + NS - 1);
    if (i < n_act) {
      __builtin_amdgcn_s_setprio(1);
      second_product(i);
      if (i + 1 < n_act) first_product(i + 1);
      __builtin_amdgcn_s_setprio(0);
    }
    __builtin_amdgcn_sched_barrier(0);
    if (group == 1) wait_tile(i + 2);
    LZ_PHASE_END();
  }
  if (group == 0) LZ_PHASE_END();
#undef LZ_LDS_READ
#undef LZ_FRAG_READY
#undef LZ_ATT_INTERLEAVE
#undef LZ_PHASE_END

  // ---- normalise and store.  Register r of block h is dim 32h + 8*(r/4) + 4*hi + r%4.
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.0f / l_tot;
  if (score_wave && qrow == n - 1 && hi == 0)
    zstat[(size_t)b * n_heads + head] = make_float2(m_run, inv);
  if (qrow < n) {
    uint16_t* op = o + (size_t)(row0 + qrow) * d + head * HD + 4 * hi;
#pragma unroll
    for (int h = 0; h < HS; ++h)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 w2;
        w2.x = pack_bf16(oacc[h][4 * g] * inv, oacc[h][4 * g + 1] * inv);
        w2.y = pack_bf16(oacc[h][4 * g + 2] * inv, oacc[h][4 * g + 3] * inv);
        *(uint2*)(op + h * 32 + 8 * g) = w2;
      }
  }
}

hipError_t launch_attention(const void* q, const void* k, const void* vt, void* o, const int32_t* cu,
                            const int32_t* cu_vt, int n_single, int batch, int max_rows, int vt_ld,
                            int n_heads, int head_dim, hipStream_t st, float* z, void* zstat,
                            int z_ld, int kv_group) {
  if (max_rows <= 0) return hipSuccess;
  if (kv_group < 1 || n_heads % kv_group != 0) return hipErrorInvalidValue;
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)head_dim);
  // 8-wave workgroups (one per CU, four stages) when they alone fill the chip: they halve the
  // L2 -> LDS traffic per query.  Otherwise 4-wave ones, which spread a short sequence over
  // more CUs.
  // (measured at 32 heads, one sequence: 1967 rows 55 us with 4 waves against 58 with 8, 2364 rows
  // 76 against 68, 3376 rows 135 against 108)
  const int nw = ((max_rows + 255) / 256) * n_heads * batch > 256 ? 8 : 4;
#define LZ_ATT(HD, NW, NS)                                                                       \
  do {                                                                                           \
    constexpr int LDS_BYTES = NS * 2 * ATT_BN * HD * 2;                                          \
    auto kern = flash_attn_kernel<HD, NW, NS>;                                                   \
    static bool attr_set = false;                                                                \
    if (!attr_set) {                                                                             \
      hipError_t e = hipFuncSetAttribute((const void*)kern,                                      \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES); \
      if (e != hipSuccess) return e;                                                             \
      attr_set = true;                                                                           \
    }                                                                                            \
    dim3 grid(n_heads, (max_rows + 32 * NW - 1) / (32 * NW), batch), block(64 * NW);             \
    hipLaunchKernelGGL(kern, grid, block, LDS_BYTES, st, (const uint16_t*)q, (const uint16_t*)k, \
                       (const uint16_t*)vt, (uint16_t*)o, cu, cu_vt, n_single, vt_ld, n_heads,   \
                       scale_log2e, z, (float2*)zstat, z_ld, kv_group);                          \
  } while (0)
  if (head_dim != 128 && head_dim != 64) return hipErrorInvalidValue;
  static const int pp_form = [] { const char* e = getenv("LAZYLLM_ATT_PP"); return e ? atoi(e) : 1; }();
#define LZ_ATT_PP(HD, NS)                                                                          \
  do {                                                                                           \
    constexpr int LDS_BYTES = NS * 2 * ATT_BN * HD * 2;                                          \
    auto kern = flash_attn_pp_kernel<HD, NS>;                                                     \
    static bool attr_set = false;                                                                \
    if (!attr_set) {                                                                             \
      hipError_t e = hipFuncSetAttribute((const void*)kern,                                      \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES); \
      if (e != hipSuccess) return e;                                                             \
      attr_set = true;                                                                           \
    }                                                                                            \
    dim3 grid(n_heads, (max_rows + 255) / 256, batch), block(512);                               \
    hipLaunchKernelGGL(kern, grid, block, LDS_BYTES, st, (const uint16_t*)q, (const uint16_t*)k, \
                       (const uint16_t*)vt, (uint16_t*)o, cu, cu_vt, n_single, vt_ld, n_heads,   \
                       scale_log2e, z, (float2*)zstat, z_ld, kv_group);                          \
  } while (0)
  // (the ping-pong form addresses a Vt tile with 32-bit lane offsets: head_dim rows of vt_ld columns)
  if (nw == 8 && pp_form && (unsigned long long)head_dim * (unsigned long long)vt_ld * 2 < (1ull << 32)) {
    if (head_dim == 128) LZ_ATT_PP(128, 4);
    else LZ_ATT_PP(64, 4);
#undef LZ_ATT_PP
    return hipGetLastError();
  }
  if (head_dim == 128 && nw == 8) LZ_ATT(128, 8, 4);
  else if (head_dim == 128) LZ_ATT(128, 4, 3);
  else if (nw == 8) LZ_ATT(64, 8, 4);
  else LZ_ATT(64, 4, 4);
#undef LZ_ATT
  return hipGetLastError();
}

}  // namespace lz
