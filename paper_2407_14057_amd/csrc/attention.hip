// Causal flash-attention prefill over the compacted token set (tokens are stored in ascending
// original position, so causality in the compacted order equals causality in the prompt).
//
// Workgroup = 4 waves = 128 queries of one head; each wave owns 32 query rows.  Keys advance
// 64 per step; the K tile [64][HD] and the transposed V tile [HD][64] are copied global -> LDS
// by global_load_lds into one of two stages.  Both products run on v_mfma_f32_32x32x16_bf16
// in the transposed orientation, so that every lane owns ONE query column:
//   S^T[key][q] = K[key][:] . Q[q][:]        A operand = K rows,   B operand = Q rows
//   O^T[dim][q] = Vt[dim][key] . P^T[key][q]  A operand = Vt rows,  B operand = P^T (registers)
// Row statistics (running max, running sum) are then per-lane scalars, and the fp32 S^T
// accumulator feeds the second product without leaving registers: the MFMA rows of S^T are
// mapped to keys through a fixed permutation (bits 2 and 3 swapped) chosen so that the 8
// accumulator values a lane holds for one 16-key step are exactly the 8 consecutive keys the
// B operand of the second product expects from that lane.
#include "common.h"

namespace lz {

constexpr int ATT_BM = 128;   // queries per workgroup
constexpr int ATT_BN = 64;    // keys per step

template <int HD>
__global__ void __launch_bounds__(256)
flash_attn_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                  const uint16_t* __restrict__ vt, uint16_t* __restrict__ o,
                  const int32_t* __restrict__ cu, const int32_t* __restrict__ cu_vt, int n_single,
                  int vt_ld, int n_heads, float scale_log2e) {
  constexpr int CHK = HD / 8;                 // 16-byte chunks per K row
  constexpr int KSTEPS = HD / 16;             // k-steps of the first product
  constexpr int HS = HD / 32;                 // 32-row blocks of O^T
  constexpr int K_TILE = ATT_BN * HD * 2;     // bytes
  constexpr int STAGE = 2 * K_TILE;           // K tile + Vt tile
  constexpr int K_INSTR = (ATT_BN * CHK / 64) / 4;   // 1 KB copies per wave for the K tile
  constexpr int V_INSTR = (HD * 8 / 64) / 4;         // ... for the Vt tile
  constexpr int K_ROWS_PER_INSTR = 64 / CHK;
  extern __shared__ __attribute__((aligned(1024))) char lds[];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int head = blockIdx.x, b = blockIdx.z;
  int row0, n;
  seq_range(cu, b, n_single, row0, n);
  const int qblocks = (n + ATT_BM - 1) / ATT_BM;
  if ((int)blockIdx.y >= qblocks) return;
  const int qb = qblocks - 1 - blockIdx.y;    // longest blocks first
  const int q0 = qb * ATT_BM;
  const int d = n_heads * HD;
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
  const uint16_t* kbase = k + (size_t)row0 * d + head * HD;
  const uint16_t* vbase = vt + (size_t)head * HD * vt_ld + (cu_vt ? cu_vt[b] : 0);
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
      g2l16(kbase + (size_t)key * d + c * 8, sk + slab * 1024);
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

  issue(0, 0);
  for (int it = 0; it < ntiles; ++it) {
    const int k0 = it * ATT_BN;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (it + 1 < ntiles) issue((it + 1) & 1, k0 + ATT_BN);
    if (k0 > q_hi) continue;                 // every key of this tile is in the future
    const char* st = lds + (it & 1) * STAGE;

    // S^T = K Q^T for the two 32-key blocks
    floatx16_t sacc[2];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[sub][r] = 0.f;
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s) {
        const bf16x8_t kf =
            *(const bf16x8_t*)(st + k_addr[sub] + (((s * 2 + hi) ^ kx) * 16));
        sacc[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], sacc[sub], 0, 0, 0);
      }
    }
    // scale, causal mask, running max.  Register r of block sub is key
    // k0 + 32*sub + 16*(r/8) + 8*hi + r%8.
    const bool need_mask = (k0 + ATT_BN - 1) > q_lo;
    float mloc = -INFINITY;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float sv = sacc[sub][r] * scale_log2e;
        if (need_mask) {
          const int key = k0 + 32 * sub + 16 * (r / 8) + 8 * hi + (r % 8);
          if (key > qrow) sv = -INFINITY;
        }
        sacc[sub][r] = sv;
        mloc = fmaxf(mloc, sv);
      }
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
    const float m_new = fmaxf(m_run, mloc);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    float psum = 0.f;
    bf16x8_t pf[2][2];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        float p[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          p[j] = __builtin_amdgcn_exp2f(sacc[sub][8 * t + j] - m_new);
          psum += p[j];
        }
        uint4 packed = pack8(p);
        pf[sub][t] = *reinterpret_cast<bf16x8_t*>(&packed);
      }
    l_run = l_run * alpha + psum;
#pragma unroll
    for (int h = 0; h < HS; ++h)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[h][r] *= alpha;
    // O^T += Vt P^T
#pragma unroll
    for (int h = 0; h < HS; ++h)
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const int chunk = sub * 4 + t * 2 + hi;
          const bf16x8_t vf =
              *(const bf16x8_t*)(st + v_addr + h * 32 * 128 + ((chunk ^ vx) * 16));
          oacc[h] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[sub][t], oacc[h], 0, 0, 0);
        }
  }

  // ---- normalise and store.  Register r of block h is dim 32h + 8*(r/4) + 4*hi + r%4.
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.0f / l_tot;
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
                            int n_heads, int head_dim, hipStream_t st) {
  if (max_rows <= 0) return hipSuccess;
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)head_dim);
  dim3 grid(n_heads, (max_rows + ATT_BM - 1) / ATT_BM, batch), block(256);
#define LZ_ATT(HD)                                                                               \
  do {                                                                                           \
    constexpr int LDS_BYTES = 2 * 2 * ATT_BN * HD * 2;                                           \
    auto kern = flash_attn_kernel<HD>;                                                           \
    static bool attr_set = false;                                                                \
    if (!attr_set) {                                                                             \
      hipError_t e = hipFuncSetAttribute((const void*)kern,                                      \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES); \
      if (e != hipSuccess) return e;                                                             \
      attr_set = true;                                                                           \
    }                                                                                            \
    hipLaunchKernelGGL(kern, grid, block, LDS_BYTES, st, (const uint16_t*)q, (const uint16_t*)k, \
                       (const uint16_t*)vt, (uint16_t*)o, cu, cu_vt, n_single, vt_ld, n_heads,   \
                       scale_log2e);                                                             \
  } while (0)
  if (head_dim == 128) LZ_ATT(128);
  else if (head_dim == 64) LZ_ATT(64);
  else return hipErrorInvalidValue;
#undef LZ_ATT
  return hipGetLastError();
}

}  // namespace lz
