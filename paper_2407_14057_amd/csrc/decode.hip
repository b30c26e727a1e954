// Decoding steps with the Aux Cache (Sec. 3.2, paragraph "Aux Cache").
//
// The generation state is indexed by ORIGINAL POSITION: per layer a K cache [capacity][d] and a
// transposed V cache [d][vt_ld], per pruning stage a byte table "K,V present" and an Aux Cache
// [capacity][d] with its own presence table.  With 288 GB of HBM a dense position-indexed cache
// is cheap (7B shape, 3.5k positions: 1.8 GB), and it removes every token->slot map: a revived
// token's K,V go to the row of its position, the causal rule is "key position <= query
// position", and the per-step selection is a bit mask over positions.
//
// Kernels here: the state's initialisation from a prefill's packed results, the new token's
// embedding, the row gather that revives tokens / parks states, and the attention of the rows
// that run a layer against the position-indexed cache under the step's selection mask.
#include "common.h"

namespace lz {

// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) fill_zero_kernel(uint4* __restrict__ p, size_t n16) {
  const uint4 z = make_uint4(0, 0, 0, 0);
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) p[i] = z;
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st) {
  if (bytes == 0) return hipSuccess;
  if ((bytes & 15) != 0 || ((uintptr_t)p & 15) != 0) return hipErrorInvalidValue;
  const size_t n16 = bytes / 16;
  const int blocks = (int)((n16 + 255) / 256 < 4096 ? (n16 + 255) / 256 : 4096);
  hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, st, (uint4*)p, n16);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Packed rows -> position-indexed rows: dst[pos[i]] = src[i], flag[pos[i]] = 1.  One wave per row.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
scatter_rows_kernel(const uint4* __restrict__ src, const int32_t* __restrict__ pos, int n,
                    uint4* __restrict__ dst, uint8_t* __restrict__ flag, int vpr) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + wave;
  if (r >= n) return;
  const int p = pos[r];
  const uint4* s = src + (size_t)r * vpr;
  uint4* d = dst + (size_t)p * vpr;
  for (int v = lane; v < vpr; v += 64) d[v] = s[v];
  if (lane == 0 && flag != nullptr) flag[p] = 1;
}

hipError_t launch_scatter_rows(const void* src, const int32_t* pos, int n, void* dst, uint8_t* flag,
                               int d, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(scatter_rows_kernel, dim3((n + 3) / 4), dim3(256), 0, st, (const uint4*)src, pos,
                     n, (uint4*)dst, flag, d / 8);
  return hipGetLastError();
}

// Packed V rows [n][d] -> transposed, position-indexed vt[f][pos[i]].  A 64-row x 64-feature
// tile goes through LDS so that the reads are whole rows and each 2-byte store instruction
// writes one feature of 64 tokens (ascending, mostly adjacent positions).
__global__ void __launch_bounds__(256)
scatter_vt_kernel(const uint16_t* __restrict__ v, const int32_t* __restrict__ pos, int n, int d,
                  uint16_t* __restrict__ vt, int vt_ld) {
  __shared__ uint16_t tile[64][66];
  const int r0 = blockIdx.x * 64, f0 = blockIdx.y * 64;
  for (int idx = threadIdx.x; idx < 64 * 8; idx += 256) {
    const int r = idx >> 3, c = idx & 7;
    uint4 x = make_uint4(0, 0, 0, 0);
    if (r0 + r < n) x = *(const uint4*)(v + (size_t)(r0 + r) * d + f0 + c * 8);
    const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      tile[r][c * 8 + 2 * e] = (uint16_t)(w[e] & 0xffff);
      tile[r][c * 8 + 2 * e + 1] = (uint16_t)(w[e] >> 16);
    }
  }
  __syncthreads();
  const int r = threadIdx.x & 63;
  if (r0 + r < n) {
    const int p = pos[r0 + r];
    for (int f = threadIdx.x >> 6; f < 64; f += 4) vt[(size_t)(f0 + f) * vt_ld + p] = tile[r][f];
  }
}

hipError_t launch_scatter_vt(const void* v, const int32_t* pos, int n, int d, void* vt, int vt_ld,
                             hipStream_t st) {
  if (n <= 0) return hipSuccess;
  if (d % 64 != 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(scatter_vt_kernel, dim3((n + 63) / 64, d / 64), dim3(256), 0, st,
                     (const uint16_t*)v, pos, n, d, (uint16_t*)vt, vt_ld);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Start of a step: the new token's embedding row (with its sum of squares for the folded
// RMSNorm), its position, and the tables that say "only the new token carries a state".
// One workgroup.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
gen_embed_kernel(const uint4* __restrict__ embed, const int32_t* __restrict__ token_id, int vocab,
                 int vpr, int new_pos, uint4* __restrict__ h, unsigned long long* __restrict__ ssq,
                 int32_t* __restrict__ run_pos, int32_t* __restrict__ live_row,
                 uint8_t* __restrict__ has_kv0, int32_t* __restrict__ status) {
  __shared__ float red[4];
  int id = token_id[0];
  if (id < 0 || id >= vocab) {
    if (threadIdx.x == 0) atomicOr(status, ST_BAD_TOKEN);
    id = id < 0 ? 0 : vocab - 1;
  }
  const uint4* src = embed + (size_t)id * vpr;
  float ss = 0.f;
  for (int v = threadIdx.x; v < vpr; v += 256) {
    const uint4 x = src[v];
    h[v] = x;
    float f[8];
    unpack8(x, f);
#pragma unroll
    for (int e = 0; e < 8; ++e) ss += f[e] * f[e];
  }
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  if (threadIdx.x == 0) {
    ssq[0] = ssq_to_fixed(red[0] + red[1] + red[2] + red[3]);
    run_pos[0] = new_pos;
    has_kv0[new_pos] = 1;
  }
  for (int i = threadIdx.x; i <= new_pos; i += 256) live_row[i] = (i == new_pos) ? 0 : -1;
}

hipError_t launch_gen_embed(const void* embed, const int32_t* token_id, int vocab, int d, int new_pos,
                            void* h, unsigned long long* ssq, int32_t* run_pos, int32_t* live_row,
                            uint8_t* has_kv0, int32_t* status, hipStream_t st) {
  hipLaunchKernelGGL(gen_embed_kernel, dim3(1), dim3(256), 0, st, (const uint4*)embed, token_id, vocab,
                     d / 8, new_pos, (uint4*)h, ssq, run_pos, live_row, has_kv0, status);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Row movement at a pruning layer of a step.  Rows 0..n_rows-1 are the tokens that run the
// layer: row r comes from row src_row[r] of the states carried out of the layer below, or,
// when src_row[r] < 0, from this layer's Aux Cache at position run_pos[r] (a revival).  The
// next n_park rows go the other way: carried states of tokens not selected here are parked
// in the Aux Cache.  One wave per row; the sum of squares of each running row is left for the
// folded RMSNorm.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
revive_gather_kernel(const uint4* __restrict__ h_prev, uint4* __restrict__ aux,
                     const int32_t* __restrict__ run_pos, const int32_t* __restrict__ src_row,
                     int n_rows, const int32_t* __restrict__ park_src,
                     const int32_t* __restrict__ park_pos, int n_park, uint4* __restrict__ h_new,
                     unsigned long long* __restrict__ ssq, int vpr) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + wave;
  if (r >= n_rows + n_park) return;
  const uint4* src;
  uint4* dst;
  const bool running = r < n_rows;
  if (running) {
    const int sr = src_row[r];
    src = sr >= 0 ? h_prev + (size_t)sr * vpr : aux + (size_t)run_pos[r] * vpr;
    dst = h_new + (size_t)r * vpr;
  } else {
    const int i = r - n_rows;
    src = h_prev + (size_t)park_src[i] * vpr;
    dst = aux + (size_t)park_pos[i] * vpr;
  }
  float ss = 0.f;
  for (int v = lane; v < vpr; v += 64) {
    const uint4 x = src[v];
    dst[v] = x;
    if (running) {
      float f[8];
      unpack8(x, f);
#pragma unroll
      for (int e = 0; e < 8; ++e) ss += f[e] * f[e];
    }
  }
  if (running) {
    ss = wave_sum(ss);
    if (lane == 0) ssq[r] = ssq_to_fixed(ss);
  }
}

hipError_t launch_revive_gather(const void* h_prev, void* aux, const int32_t* run_pos,
                                const int32_t* src_row, int n_rows, const int32_t* park_src,
                                const int32_t* park_pos, int n_park, void* h_new,
                                unsigned long long* ssq, int d, hipStream_t st) {
  const int rows = n_rows + n_park;
  if (rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(revive_gather_kernel, dim3((rows + 3) / 4), dim3(256), 0, st,
                     (const uint4*)h_prev, (uint4*)aux, run_pos, src_row, n_rows, park_src, park_pos,
                     n_park, (uint4*)h_new, ssq, d / 8);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Attention of the rows that run a layer in a decoding step.  Queries: M rows (ascending
// position qpos[]; the last one is the step's new token).  Keys: the position-indexed cache,
// positions 0..n_keys-1, of which only those selected in this step take part (bit p of
// sel_bits, all when null) and, per query, only those at or before its own position.
//
// Same transposed MFMA formulation as the prefill kernel (S^T = K Q^T, O^T = Vt P^T, a lane
// owns one query, key rows permuted so that the S^T accumulator is the second product's B
// operand), with 4 waves of 32 queries, 64 keys per step, two LDS stages and one barrier per
// step: a decoding step's attention is small next to its projections, so this kernel is kept
// simple.  The new token's logits (base-2 domain, -inf for keys that take no part) and its
// (max, 1/sum) go to z / zstat for Eq. 1, as in the prefill.
// ------------------------------------------------------------------------------------------
template <int HD>
__global__ void __launch_bounds__(256)
decode_attn_kernel(const uint16_t* __restrict__ q, const int32_t* __restrict__ qpos, int M,
                   const uint16_t* __restrict__ k, const uint16_t* __restrict__ vt, int vt_ld,
                   const unsigned long long* __restrict__ sel_bits, int n_keys,
                   uint16_t* __restrict__ o, int n_heads, float scale_log2e, float* __restrict__ z,
                   float2* __restrict__ zstat, int z_ld, int n_splits, float* __restrict__ po,
                   float2* __restrict__ pml, int kv_group) {
  constexpr int NW = 4, BN = 64;
  constexpr int CHK = HD / 8, KSTEPS = HD / 16, HS = HD / 32;
  constexpr int K_TILE = BN * HD * 2, STAGE = 2 * K_TILE;
  constexpr int K_INSTR = (BN * CHK / 64) / NW, V_INSTR = (HD * 8 / 64) / NW;
  constexpr int K_ROWS_PER_INSTR = 64 / CHK;
  extern __shared__ __attribute__((aligned(1024))) char lds[];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int head = blockIdx.x;
  const int q0 = blockIdx.y * (32 * NW);
  const int d = n_heads * HD;
  const int kvd = d / kv_group, kvh = head / kv_group;      // grouped-query attention: shared K,V heads
  const int hi = lane >> 5, l31 = lane & 31;
  const int qrow = q0 + wave * 32 + l31;
  const int qrow_c = qrow < M ? qrow : M - 1;
  const int my_pos = qpos[qrow_c];
  const int blk_last = (q0 + 32 * NW < M ? q0 + 32 * NW : M) - 1;
  const int ntiles_blk = qpos[blk_last] / BN + 1;           // keys 0 .. the block's last position
  // with few queries the keys are split over blockIdx.z: each split leaves (max, sum, unnormalised
  // output) per query and a second kernel merges them
  const int sp = blockIdx.z;
  const int per_split = (ntiles_blk + n_splits - 1) / n_splits;
  const int t_lo = sp * per_split;
  const int t_hi = min(t_lo + per_split, ntiles_blk);
  const int w_first = q0 + wave * 32;
  const int w_last = w_first + 31 < M ? w_first + 31 : M - 1;
  const int wave_max_pos = w_first < M ? qpos[w_last] : -1; // -1: this wave has no query

  bf16x8_t qf[KSTEPS];
  {
    const uint16_t* qp = q + (size_t)qrow_c * d + head * HD + hi * 8;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) qf[s] = *(const bf16x8_t*)(qp + s * 16);
  }

  const uint16_t* kbase = k + kvh * HD;
  const uint16_t* vbase = vt + (size_t)kvh * HD * vt_ld;
  auto issue = [&](int stage, int k0) {
    char* sk = lds + stage * STAGE;
    char* sv = sk + K_TILE;
#pragma unroll
    for (int qi = 0; qi < K_INSTR; ++qi) {
      const int slab = wave * K_INSTR + qi;
      const int r = slab * K_ROWS_PER_INSTR + lane / CHK;
      const int c = (lane % CHK) ^ (CHK == 16 ? swz128(r) : swz64(r));
      int key = k0 + r;
      key = key < n_keys ? key : n_keys - 1;
      g2l16(kbase + (size_t)key * kvd + c * 8, sk + slab * 1024);
    }
#pragma unroll
    for (int qi = 0; qi < V_INSTR; ++qi) {
      const int slab = wave * V_INSTR + qi;
      const int r = slab * 8 + (lane >> 3);
      const int c = (lane & 7) ^ swz64(r);
      g2l16(vbase + (size_t)r * vt_ld + k0 + c * 8, sv + slab * 1024);
    }
  };

  const int kperm = (l31 & 0x13) | ((l31 & 4) << 1) | ((l31 & 8) >> 1);   // swap bits 2 and 3
  uint32_t k_addr[2];
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) k_addr[sub] = (uint32_t)((sub * 32 + kperm) * HD * 2);
  const int kx = CHK == 16 ? swz128(kperm) : swz64(kperm);
  const uint32_t v_addr = (uint32_t)(K_TILE + l31 * 128);
  const int vx = swz64(l31);
  auto kread = [&](const char* st, int sub, int s) {
    return *(const bf16x8_t*)(st + k_addr[sub] + (((s * 2 + hi) ^ kx) * 16));
  };
  auto vread = [&](const char* st, int i) {
    const int chunk = ((i >> 1) & 1) * 4 + (i & 1) * 2 + hi;
    return *(const bf16x8_t*)(st + v_addr + (i >> 2) * 32 * 128 + ((chunk ^ vx) * 16));
  };

  floatx16_t oacc[HS];
#pragma unroll
  for (int h = 0; h < HS; ++h)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[h][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const bool score_lane = z != nullptr && qrow == M - 1;

  if (t_lo < t_hi) issue(0, t_lo * BN);
  for (int it = t_lo; it < t_hi; ++it) {
    const int k0 = it * BN;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();           // tile `it` has landed for every wave; everyone is done with tile it-1
    if (it + 1 < t_hi) issue((it + 1 - t_lo) & 1, k0 + BN);
    if (k0 > wave_max_pos) continue;                        // (uniform per wave; barriers stay matched)
    const char* st = lds + ((it - t_lo) & 1) * STAGE;
    floatx16_t sacc[2];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[sub][r] = 0.f;
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s)
        sacc[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kread(st, sub, s), qf[s], sacc[sub], 0, 0, 0);
    }
    // keys of this step that take part at all (selected, inside the sequence) ...
    unsigned long long word = sel_bits != nullptr ? sel_bits[it] : ~0ull;
    if (k0 + BN > n_keys) word &= (1ull << (n_keys - k0)) - 1ull;
    const unsigned long long wsh = word >> (8 * hi);
    // ... and, per query, those not after it.  Register r of block sub is key
    // k0 + 32*sub + 16*(r/8) + 8*hi + r%8.
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int bit = 32 * sub + 16 * (r / 8) + (r % 8);
        const int key = k0 + bit + 8 * hi;
        const bool vis = ((wsh >> bit) & 1ull) != 0 && key <= my_pos;
        if (!vis) sacc[sub][r] = -INFINITY;
      }
    if (score_lane) {
      float* zr = z + (size_t)head * z_ld + k0 + 8 * hi;
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
    float mloc = -INFINITY;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int r = 0; r < 16; ++r) mloc = fmaxf(mloc, sacc[sub][r]);
    mloc *= scale_log2e;
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
    // a query may see nothing in its first steps: keep the reference point finite then
    const float m_new = fmaxf(m_run, mloc);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
    m_run = m_new;
    l_run *= alpha;
#pragma unroll
    for (int h = 0; h < HS; ++h) oacc[h] *= alpha;
    bf16x8_t pf[2][2];
    float psum = 0.f;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        float p[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          p[j] = __builtin_amdgcn_exp2f(fmaf(sacc[sub][8 * t + j], scale_log2e, -m_use));
          psum += p[j];
        }
        uint4 packed = pack8(p);
        pf[sub][t] = *reinterpret_cast<bf16x8_t*>(&packed);
      }
    l_run += psum;
#pragma unroll
    for (int i = 0; i < 2 * KSTEPS; ++i)
      oacc[i >> 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vread(st, i), pf[(i >> 1) & 1][i & 1],
                                                             oacc[i >> 2], 0, 0, 0);
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (n_splits > 1) {
    if (qrow < M) {
      if (hi == 0) pml[((size_t)sp * M + qrow) * n_heads + head] = make_float2(m_run, l_tot);
      float* pp = po + ((size_t)sp * M + qrow) * d + head * HD + 4 * hi;
#pragma unroll
      for (int h = 0; h < HS; ++h)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float4 v4 = {oacc[h][4 * g], oacc[h][4 * g + 1], oacc[h][4 * g + 2], oacc[h][4 * g + 3]};
          *(float4*)(pp + h * 32 + 8 * g) = v4;
        }
    }
    return;
  }
  const float inv = 1.0f / l_tot;
  if (score_lane && hi == 0) zstat[head] = make_float2(m_run, inv);
  if (qrow < M) {
    uint16_t* op = o + (size_t)qrow * d + head * HD + 4 * hi;
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
// Attention of a step in which only the new token runs the layer (no revived rows): one query
// per head against the selected keys.  There is no contraction to speak of, the kernel is a
// stream of the K,V cache, so it uses no MFMA and no LDS staging.  A wave takes 64 keys at a
// time (one word of the selection mask): 16-byte loads, HD/8 lanes per key row of K and 8 lanes
// per dimension row of V^T, all of a chunk's loads in flight before the first use; rows of K
// whose key takes no part are not read.  The G query heads that share a K,V head are served by
// the same loads.  Scores move from "lanes of a key" to "lane = key" through a wave-private LDS
// row, the probabilities move back the same way.  The 4 waves of a workgroup interleave the
// chunks of the workgroup's key range and are merged through LDS; key ranges (blockIdx.y, at
// most 16) are merged by the workgroup that finishes last.  `counters` (one per K,V head) must
// be zero on entry and are zero again on exit.
// ------------------------------------------------------------------------------------------
template <int HD, int G>
__global__ void __launch_bounds__(256)
decode_attn1_kernel(const uint16_t* __restrict__ q, const int32_t* __restrict__ qpos,
                    const uint16_t* __restrict__ k, const uint16_t* __restrict__ vt, int vt_ld,
                    const unsigned long long* __restrict__ sel_bits, int n_keys,
                    uint16_t* __restrict__ o, int n_heads, float scale_log2e, float* __restrict__ z,
                    float2* __restrict__ zstat, int z_ld, int n_splits, float* __restrict__ po,
                    float2* __restrict__ pml, unsigned* __restrict__ counters) {
  constexpr int CHK = HD / 8;        // lanes per key row of K (16 bytes each)
  constexpr int KPI = 64 / CHK;      // keys per K load instruction
  constexpr int NKI = CHK;           // K load instructions per 64 keys
  constexpr int NVI = HD / 8;        // V^T load instructions per 64 keys (8 dimension rows each)
  __shared__ float sc[4][G][64];
  __shared__ float mo[4][G][HD + 2];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int kvh = blockIdx.x, sp = blockIdx.y;
  const int d = n_heads * HD, kvd = d / G;
  const int my_pos = qpos[0];
  const int n_vis = min(n_keys, my_pos + 1);                 // keys 0 .. n_vis-1 can be seen at all
  const int chunks = (n_vis + 63) / 64;
  const int per_split = (chunks + n_splits - 1) / n_splits;
  const int c_lo = sp * per_split, c_hi = min(c_lo + per_split, chunks);
  const int kl = lane % CHK, kg = lane / CHK;

  float qf[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g)
    unpack8(*(const uint4*)(q + (size_t)(kvh * G + g) * HD + kl * 8), qf[g]);
  float acc[G][NVI], m_run[G], l_run[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m_run[g] = -INFINITY;
    l_run[g] = 0.f;
#pragma unroll
    for (int i = 0; i < NVI; ++i) acc[g][i] = 0.f;
  }
  const uint16_t* kbase = k + (size_t)kvh * HD + kl * 8;
  const uint16_t* vbase = vt + ((size_t)kvh * HD + (lane >> 3)) * vt_ld + (lane & 7) * 8;

  for (int c = c_lo + wave; c < c_hi; c += 4) {
    const int k0 = c * 64;
    unsigned long long word = sel_bits != nullptr ? sel_bits[c] : ~0ull;
    if (k0 + 64 > n_vis) word &= (1ull << (n_vis - k0)) - 1ull;
    uint4 kr[NKI], vr[NVI];
#pragma unroll
    for (int i = 0; i < NKI; ++i) {
      const int j = i * KPI + kg;
      kr[i] = make_uint4(0u, 0u, 0u, 0u);
      if ((word >> j) & 1ull) kr[i] = *(const uint4*)(kbase + (size_t)(k0 + j) * kvd);
    }
#pragma unroll
    for (int i = 0; i < NVI; ++i) vr[i] = *(const uint4*)(vbase + (size_t)i * 8 * vt_ld + k0);
    // scores: each lane's 8 dimensions, then a sum over the CHK lanes of a key
#pragma unroll
    for (int i = 0; i < NKI; ++i) {
      float kf[8];
      unpack8(kr[i], kf);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) s = fmaf(kf[e], qf[g][e], s);
#pragma unroll
        for (int off = 1; off < CHK; off <<= 1) s += __shfl_xor(s, off, 64);
        if (kl == 0) sc[wave][g][i * KPI + kg] = s;
      }
    }
    __builtin_amdgcn_wave_barrier();
    const bool vis = ((word >> lane) & 1ull) != 0;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float s = vis ? sc[wave][g][lane] * scale_log2e : -INFINITY;
      if (z != nullptr) z[(size_t)(kvh * G + g) * z_ld + k0 + lane] = s;
      const float m_new = fmaxf(m_run[g], wave_max(s));
      const float m_use = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run[g] - m_use);
      const float p = __builtin_amdgcn_exp2f(s - m_use);
      m_run[g] = m_new;
      l_run[g] = l_run[g] * alpha + p;
#pragma unroll
      for (int i = 0; i < NVI; ++i) acc[g][i] *= alpha;
      sc[wave][g][lane] = p;
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float4 p0 = *(const float4*)&sc[wave][g][(lane & 7) * 8];
      const float4 p1 = *(const float4*)&sc[wave][g][(lane & 7) * 8 + 4];
      const float pp[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
#pragma unroll
      for (int i = 0; i < NVI; ++i) {
        float vf[8];
        unpack8(vr[i], vf);
        float a = acc[g][i];
#pragma unroll
        for (int e = 0; e < 8; ++e) a = fmaf(vf[e], pp[e], a);
        acc[g][i] = a;
      }
    }
    __builtin_amdgcn_wave_barrier();                         // the next chunk overwrites sc
  }

  // per wave: finish the sums over lanes and leave (output, max, sum) in LDS
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const float l = wave_sum(l_run[g]);
#pragma unroll
    for (int i = 0; i < NVI; ++i) {
      float a = acc[g][i];
      a += __shfl_xor(a, 1, 64);
      a += __shfl_xor(a, 2, 64);
      a += __shfl_xor(a, 4, 64);
      if ((lane & 7) == 0) mo[wave][g][i * 8 + (lane >> 3)] = a;
    }
    if (lane == 0) {
      mo[wave][g][HD] = m_run[g];
      mo[wave][g][HD + 1] = l;
    }
  }
  __syncthreads();
  // the workgroup's 4 waves, merged: thread -> (head g, dimension)
  constexpr int NPASS = (G * HD + 255) / 256;
  float ov[NPASS], lv[NPASS], mv[NPASS];
#pragma unroll
  for (int ps = 0; ps < NPASS; ++ps) {
    const int idx = ps * 256 + threadIdx.x;
    const int g = idx < G * HD ? idx / HD : 0, dim = idx % HD;
    float m = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) m = fmaxf(m, mo[w][g][HD]);
    float a = 0.f, l = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float mw = mo[w][g][HD];
      const float f = mw == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mw - m);
      a += f * mo[w][g][dim];
      l += f * mo[w][g][HD + 1];
    }
    ov[ps] = a; lv[ps] = l; mv[ps] = m;
  }
  if (n_splits > 1) {
    // Key ranges over workgroups: every workgroup leaves (output, max, sum) in the workspace and
    // draws a ticket from its K,V head's counter; the one that draws the last ticket merges all
    // ranges in range order and resets the counter.  Partial results are written with
    // agent-scope atomic stores and read with agent-scope atomic loads (both bypass the
    // non-coherent caches), so that no release fence -- a write-back of the whole L2 -- is needed;
    // the stores have completed (vmcnt) before the ticket is drawn.
    __shared__ unsigned last_flag;
    float* pmlf = (float*)pml;
#pragma unroll
    for (int ps = 0; ps < NPASS; ++ps) {
      const int idx = ps * 256 + threadIdx.x;
      if (idx < G * HD) {
        const int head = kvh * G + idx / HD, dim = idx % HD;
        __hip_atomic_store(po + (size_t)sp * d + head * HD + dim, ov[ps], __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
        if (dim == 0) {
          __hip_atomic_store(pmlf + 2 * ((size_t)sp * n_heads + head), mv[ps], __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_store(pmlf + 2 * ((size_t)sp * n_heads + head) + 1, lv[ps], __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
        }
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0)
      last_flag = __hip_atomic_fetch_add(counters + kvh, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                          (unsigned)(n_splits - 1) ? 1u : 0u;
    __syncthreads();
    if (last_flag == 0) return;
#pragma unroll
    for (int ps = 0; ps < NPASS; ++ps) {
      const int idx = ps * 256 + threadIdx.x;
      const int head = kvh * G + (idx < G * HD ? idx / HD : 0), dim = idx % HD;
      float ms[16], ls[16], os[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const bool on = u < n_splits;
        ms[u] = on ? __hip_atomic_load(pmlf + 2 * ((size_t)u * n_heads + head), __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT) : -INFINITY;
        ls[u] = on ? __hip_atomic_load(pmlf + 2 * ((size_t)u * n_heads + head) + 1, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT) : 0.f;
        os[u] = on ? __hip_atomic_load(po + (size_t)u * d + head * HD + dim, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT) : 0.f;
      }
      float m = -INFINITY;
#pragma unroll
      for (int u = 0; u < 16; ++u) m = fmaxf(m, ms[u]);
      float a = 0.f, l = 0.f;
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const float f = ms[u] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ms[u] - m);
        a += f * os[u];
        l += f * ls[u];
      }
      ov[ps] = a; lv[ps] = l; mv[ps] = m;
    }
    if (threadIdx.x == 0) counters[kvh] = 0;                 // ready for the next launch
  }
#pragma unroll
  for (int ps = 0; ps < NPASS; ++ps) {
    const int idx = ps * 256 + threadIdx.x;
    if (idx < G * HD) {
      const int head = kvh * G + idx / HD, dim = idx % HD;
      const float inv = 1.0f / lv[ps];
      o[head * HD + dim] = to_bf16(ov[ps] * inv);
      if (dim == 0 && zstat != nullptr) zstat[head] = make_float2(mv[ps], inv);
    }
  }
}

// Merges the key splits of decode_attn_kernel: per (query, head) the splits' (max m_s, sum l_s,
// unnormalised output o_s) combine as o = sum_s 2^(m_s - m) o_s / sum_s 2^(m_s - m) l_s with
// m = max_s m_s, splits added in order.  One thread per output dimension.
__global__ void __launch_bounds__(128)
decode_attn_merge_kernel(const float* __restrict__ po, const float2* __restrict__ pml, int n_splits,
                         int M, int n_heads, int hd, uint16_t* __restrict__ o,
                         float2* __restrict__ zstat) {
  const int row = blockIdx.x, head = blockIdx.y, dim = threadIdx.x;
  if (dim >= hd) return;
  const int d = n_heads * hd;
  float m = -INFINITY;
  for (int s = 0; s < n_splits; ++s) m = fmaxf(m, pml[((size_t)s * M + row) * n_heads + head].x);
  float l = 0.f, acc = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    const float2 ml = pml[((size_t)s * M + row) * n_heads + head];
    const float w = ml.x == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ml.x - m);
    l += w * ml.y;
    acc += w * po[((size_t)s * M + row) * d + head * hd + dim];
  }
  const float inv = 1.0f / l;
  o[(size_t)row * d + head * hd + dim] = to_bf16(acc * inv);
  if (zstat != nullptr && row == M - 1 && dim == 0) zstat[head] = make_float2(m, inv);
}

constexpr size_t DATT_COUNTER_BYTES = 4096;       // one ticket counter per K,V head

size_t decode_attention_workspace_bytes(int d_model, int n_heads) {
  // 16 splits of up to 128 queries: fp32 outputs and (max, sum) pairs; then the one-query
  // kernel's ticket counters
  return (size_t)16 * 128 * ((size_t)d_model * 4 + (size_t)n_heads * 8) + DATT_COUNTER_BYTES;
}

hipError_t launch_decode_attention_counters_clear(void* split_ws, size_t split_ws_bytes, hipStream_t st) {
  if (split_ws == nullptr || split_ws_bytes < DATT_COUNTER_BYTES) return hipErrorInvalidValue;
  return launch_fill_zero((char*)split_ws + split_ws_bytes - DATT_COUNTER_BYTES, DATT_COUNTER_BYTES, st);
}

hipError_t launch_decode_attention(const void* q, const int32_t* qpos, int M, const void* k,
                                   const void* vt, int vt_ld, const unsigned long long* sel_bits,
                                   int n_keys, void* o, int n_heads, int head_dim, hipStream_t st,
                                   float* z, void* zstat, int z_ld, void* split_ws,
                                   size_t split_ws_bytes, int kv_group) {
  if (M <= 0 || n_keys <= 0) return hipErrorInvalidValue;
  if (kv_group < 1 || n_heads % kv_group != 0) return hipErrorInvalidValue;
  if (head_dim != 128 && head_dim != 64) return hipErrorInvalidValue;
  if (vt_ld < (n_keys + 63) / 64 * 64) return hipErrorInvalidValue;
  if (z != nullptr && (zstat == nullptr || z_ld < (n_keys + 63) / 64 * 64)) return hipErrorInvalidValue;
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)head_dim);
  unsigned* counters = nullptr;                      // (the one-query kernel's tickets: end of the workspace)
  if (split_ws != nullptr) {
    if (split_ws_bytes < DATT_COUNTER_BYTES || (size_t)(n_heads / kv_group) * 4 > DATT_COUNTER_BYTES)
      return hipErrorInvalidValue;
    split_ws_bytes -= DATT_COUNTER_BYTES;
    counters = (unsigned*)((char*)split_ws + split_ws_bytes);
  }
  // A step's queries (the new token and the revived ones) make few workgroups: split the keys so
  // that about 512 are in flight, each with at least two key tiles, as far as the workspace for
  // the splits' partial results reaches.
  const int qblocks = (M + 127) / 128, d_model = n_heads * head_dim;
  int n_splits = 1;
  if (split_ws != nullptr) {
    const int tiles = (n_keys + 63) / 64;
    n_splits = 512 / (n_heads * qblocks);
    if (n_splits > tiles / 2) n_splits = tiles / 2;
    if (n_splits > 16) n_splits = 16;
    const size_t per_split = (size_t)M * ((size_t)d_model * 4 + (size_t)n_heads * 8);
    while (n_splits > 1 && (size_t)n_splits * per_split > split_ws_bytes) --n_splits;
    if (n_splits < 1) n_splits = 1;
  }
  // only the new token runs the layer: the streaming kernel, about four 64-key chunks per workgroup
  const bool one_query = M == 1 && split_ws != nullptr && (kv_group == 1 || kv_group == 2 || kv_group == 4);
  if (one_query) {
    const int chunks = (n_keys + 63) / 64;
    n_splits = (chunks + 3) / 4;
    if (n_splits > 16) n_splits = 16;
    const size_t per_split = (size_t)d_model * 4 + (size_t)n_heads * 8;
    while (n_splits > 1 && (size_t)n_splits * per_split > split_ws_bytes) --n_splits;
  }
  float* po = (float*)split_ws;
  float2* pml = (float2*)((char*)split_ws + (size_t)n_splits * M * d_model * 4);
  if (one_query) {
    dim3 grid1(n_heads / kv_group, n_splits);
#define LZ_DATT1(HD, G)                                                                            \
  hipLaunchKernelGGL((decode_attn1_kernel<HD, G>), grid1, dim3(256), 0, st, (const uint16_t*)q, qpos, \
                     (const uint16_t*)k, (const uint16_t*)vt, vt_ld, sel_bits, n_keys, (uint16_t*)o, \
                     n_heads, scale_log2e, z, (float2*)zstat, z_ld, n_splits, po, pml, counters)
    if (head_dim == 128) {
      if (kv_group == 1) LZ_DATT1(128, 1);
      else if (kv_group == 2) LZ_DATT1(128, 2);
      else LZ_DATT1(128, 4);
    } else {
      if (kv_group == 1) LZ_DATT1(64, 1);
      else if (kv_group == 2) LZ_DATT1(64, 2);
      else LZ_DATT1(64, 4);
    }
#undef LZ_DATT1
    return hipGetLastError();
  }
  dim3 grid(n_heads, qblocks, n_splits), block(256);
#define LZ_DATT(HD)                                                                                \
  do {                                                                                             \
    constexpr int LDS_BYTES = 2 * 2 * 64 * HD * 2;                                                 \
    auto kern = decode_attn_kernel<HD>;                                                            \
    static bool attr_set = false;                                                                  \
    if (!attr_set) {                                                                               \
      hipError_t e = hipFuncSetAttribute((const void*)kern,                                        \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);   \
      if (e != hipSuccess) return e;                                                               \
      attr_set = true;                                                                             \
    }                                                                                              \
    hipLaunchKernelGGL(kern, grid, block, LDS_BYTES, st, (const uint16_t*)q, qpos, M,              \
                       (const uint16_t*)k, (const uint16_t*)vt, vt_ld, sel_bits, n_keys,           \
                       (uint16_t*)o, n_heads, scale_log2e, z, (float2*)zstat, z_ld, n_splits, po,  \
                       pml, kv_group);                                                             \
  } while (0)
  if (head_dim == 128) LZ_DATT(128);
  else LZ_DATT(64);
#undef LZ_DATT
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || n_splits == 1) return e;
  hipLaunchKernelGGL(decode_attn_merge_kernel, dim3(M, n_heads), dim3(128), 0, st, po, pml, n_splits, M,
                     n_heads, head_dim, (uint16_t*)o, z != nullptr ? (float2*)zstat : nullptr);
  return hipGetLastError();
}

}  // namespace lz
