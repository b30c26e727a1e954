// Pieces shared by the 16-bit and the 8-bit tile kernels: the workgroup -> tile map, what happens to
// a wave's TM x TN accumulator blocks after the K loop (the epilogues), and the tile's way out
// through LDS.
#pragma once
#include "common.h"

namespace lz {

constexpr int BK = 64;                 // K elements per step = 128 bytes = 8 chunks per row
constexpr int ROW_BYTES = BK * 2;

// ---- epilogue.  The W rows are the MFMA's row operand, so each 32x32 block holds C
// transposed: lane l owns token (l & 31); its register r is output feature
// 8*(r/4) + 4*(l>>5) + r%4.  Four consecutive features pack into one 8-byte store.
//
// EPI_QKV_ROPE: the N axis is [q | k | v] of width d each.  A wave's TN*32 columns hold whole
// heads, so the rotary partner of dimension i (i + hd/2) is the same register of block j + hd/64:
// q and k are rotated in fp32 straight out of the accumulator and rounded to bf16 once.
// 1/rms of this lane's TM token rows, fetched before the main loop so that the epilogue does not
// wait for it (rows past M get 0).
template <int TM>
__device__ __forceinline__ void load_row_scales(float (&rs)[TM], const EpiArgs& ra, int M, int m0,
                                                int wm, int lane) {
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int row = m0 + (wm * TM + i) * 32 + (lane & 31);
    rs[i] = (ra.ssq_in != nullptr && row < M)
                ? rsqrtf((float)ra.ssq_in[ra.a_rows != nullptr ? ra.a_rows[row] : row] * ra.ssq_mul + ra.eps)
                : 0.f;
  }
}

// Staged output: the epilogue writes the tile row-major into LDS (free after the K loop) and the
// workgroup then copies it out with 16-byte stores that cover whole 128-byte lines.  Straight from
// the MFMA layout a store instruction's 64 lanes hit 64 different rows, i.e. 64 separate lines:
// that costs 5-11 us per round of 256x256 tiles (measured by leaving the stores out).
// Layout: rows of NCH 16-byte chunks, chunk c of row r at slot c ^ (r & (NCH-1)): the 32 lanes
// that write one column block of 32 rows and the lanes that read one row both spread over the banks.
template <int NCH>
__device__ __forceinline__ uint32_t stage_off(int r, int c) {      // c: element column, multiple of 4
  return (uint32_t)(r * (NCH * 16) + (((c >> 3) ^ (r & (NCH - 1))) << 4) + ((c & 7) << 1));
}

template <int TM, int TN, int EPI, bool STAGED = false, int NCH = 32>
__device__ __forceinline__ void gemm_epilogue(floatx16_t (&acc)[TM][TN], uint16_t* __restrict__ C,
                                              const uint16_t* __restrict__ R, int M, int ldc,
                                              int m0, int n0, int wm, int wn, int lane,
                                              const EpiArgs& ra, const float* rs_pre = nullptr,
                                              char* sl = nullptr) {
  const int tok_l = lane & 31, feat_l = 4 * (lane >> 5);
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int row = m0 + (wm * TM + i) * 32 + tok_l;
    const bool valid = row < M;
    if (ra.ssq_clear != nullptr && n0 == 0 && wn == 0 && lane < 32 && valid) ra.ssq_clear[row] = 0;
    if (EPI != EPI_RESIDUAL && ra.ssq_in != nullptr) {
      // RMSNorm of the A operand's row, applied to the product
      const float rs = rs_pre != nullptr ? rs_pre[i]
                       : valid ? rsqrtf((float)ra.ssq_in[ra.a_rows != nullptr ? ra.a_rows[row] : row] *
                                            ra.ssq_mul + ra.eps) : 0.f;
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[i][j] *= rs;
    }
    if (EPI != EPI_QKV_ROPE64 && EPI != EPI_QKV_ROPE128 && !valid) continue;
    if (EPI == EPI_QKV_ROPE64 || EPI == EPI_QKV_ROPE128) {
      constexpr int hd = (EPI == EPI_QKV_ROPE64) ? 64 : 128, half = hd >> 1;
      // columns [0, d) are q, then kvd of k and kvd of v (kvd = d unless K,V heads are shared by
      // groups of query heads); rows of q are d wide, rows of k and v kvd
      const int d = ra.d_model, kvd = ra.kv_dim > 0 ? ra.kv_dim : d;
      const int col0 = n0 + wn * TN * 32;              // first column of this wave
      const int region = col0 < d ? 0 : col0 < d + kvd ? 1 : 2;   // q, k, v (uniform per wave)
      const int rcol0 = col0 - (region == 0 ? 0 : region == 1 ? d : d + kvd);
      const int rld = region == 0 ? d : kvd;
      if (region != 2 && !valid) continue;              // (the V branch keeps every lane: lane pairs exchange data)
      const int orow = (region == 1 && ra.k_row != nullptr && valid) ? ra.k_row[row] : row;
      uint16_t* dst = (region == 0 ? ra.q : region == 1 ? ra.k : ra.v) + (size_t)orow * rld +
                      rcol0 + feat_l;
      if (region == 2) {
        // V goes to the KV cache row-major and, for the attention kernel's second product,
        // transposed: a register holds one feature of 32 consecutive tokens across lanes, so
        // each 2-byte store instruction writes 64 contiguous bytes of a feature row.
        uint16_t* vtp = nullptr;
        int vcol = 0;
        if (ra.vt != nullptr && valid) {
          vcol = ra.vt_col != nullptr ? ra.vt_col[row] : row;
          vtp = ra.vt + (size_t)(rcol0 + feat_l) * ra.vt_ld + vcol;
        }
        // Neighbouring lanes hold neighbouring tokens: lane pairs swap one value each so that an
        // even lane writes tokens (t, t+1) of one feature and the odd lane (t-1, t) of the next
        // feature, 4 bytes per lane.  Needs the even lane's column to be even and both tokens
        // to be in the same sequence and below M; otherwise 2-byte stores.
        const int partner_col = __shfl_xor(vtp != nullptr ? vcol : -7, 1, 64);
        const bool odd = lane & 1;
        const bool paired = vtp != nullptr &&
                            partner_col == (odd ? vcol - 1 : vcol + 1) && (((odd ? vcol - 1 : vcol) & 1) == 0);
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            uint2 w2;
            w2.x = pack_bf16(acc[i][j][4 * g], acc[i][j][4 * g + 1]);
            w2.y = pack_bf16(acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
            if (STAGED) {
              *(uint2*)(sl + stage_off<NCH>((wm * TM + i) * 32 + tok_l,
                                            (wn * TN + j) * 32 + 8 * g + feat_l)) = w2;
            } else if (valid && ra.v != nullptr) {
              *(uint2*)(dst + j * 32 + 8 * g) = w2;
            }
            // features 8g..8g+3 of this token: w2.x = (f0, f1), w2.y = (f2, f3)
            // even lane sends (f1, f3), receives partner's (f0, f2); odd lane the other way
            const uint32_t mine_lo = (w2.x & 0xffff) | (w2.y << 16);        // (f0, f2)
            const uint32_t mine_hi = (w2.x >> 16) | (w2.y & 0xffff0000u);   // (f1, f3)
            const uint32_t got = (uint32_t)__builtin_amdgcn_mov_dpp((int)(odd ? mine_lo : mine_hi),
                                                                    0xB1, 0xf, 0xf, true);
            if (paired) {
              // even lane: features f0, f2 of tokens (t, t+1); odd lane: f1, f3 of (t-1, t)
              uint16_t* f0 = vtp + (size_t)(j * 32 + 8 * g + (odd ? 1 : 0)) * ra.vt_ld - (odd ? 1 : 0);
              const uint32_t own = odd ? mine_hi : mine_lo;
              const uint32_t a = odd ? ((got & 0xffff) | (own << 16)) : ((own & 0xffff) | (got << 16));
              const uint32_t c = odd ? ((got >> 16) | (own & 0xffff0000u)) : ((own >> 16) | (got & 0xffff0000u));
              *(uint32_t*)f0 = a;
              *(uint32_t*)(f0 + 2 * (size_t)ra.vt_ld) = c;
            } else if (vtp != nullptr) {
              uint16_t* f0 = vtp + (size_t)(j * 32 + 8 * g) * ra.vt_ld;
              f0[0] = (uint16_t)(w2.x & 0xffff);
              f0[(size_t)ra.vt_ld] = (uint16_t)(w2.x >> 16);
              f0[2 * (size_t)ra.vt_ld] = (uint16_t)(w2.y & 0xffff);
              f0[3 * (size_t)ra.vt_ld] = (uint16_t)(w2.y >> 16);
            }
          }
      } else {
        constexpr int P = hd >> 6;                      // blocks per half head: 1 (hd 64) or 2 (hd 128)
        const float2* cs = ra.table + (size_t)ra.pos[row] * half + feat_l;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          if ((j / P) & 1) continue;                    // second halves are written with their partner
          if (j + P >= TN) continue;
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const float2* t = cs + (j % P) * 32 + 8 * g;
            const float4 t01 = *(const float4*)t, t23 = *(const float4*)(t + 2);
            const float c[4] = {t01.x, t01.z, t23.x, t23.z}, sn[4] = {t01.y, t01.w, t23.y, t23.w};
            float lo[4], hi[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float x1 = acc[i][j][4 * g + e], x2 = acc[i][j + P][4 * g + e];
              lo[e] = x1 * c[e] - x2 * sn[e];
              hi[e] = x2 * c[e] + x1 * sn[e];
            }
            uint2 w2, w3;
            w2.x = pack_bf16(lo[0], lo[1]); w2.y = pack_bf16(lo[2], lo[3]);
            w3.x = pack_bf16(hi[0], hi[1]); w3.y = pack_bf16(hi[2], hi[3]);
            if (STAGED) {
              const int rl = (wm * TM + i) * 32 + tok_l, cl = (wn * TN + j) * 32 + 8 * g + feat_l;
              *(uint2*)(sl + stage_off<NCH>(rl, cl)) = w2;
              *(uint2*)(sl + stage_off<NCH>(rl, cl + P * 32)) = w3;
            } else {
              *(uint2*)(dst + j * 32 + 8 * g) = w2;
              *(uint2*)(dst + (j + P) * 32 + 8 * g) = w3;
            }
          }
        }
      }
    } else if (EPI == EPI_SWIGLU) {
#pragma unroll
      for (int j = 0; j < TN; j += 2) {            // block j = gate, block j+1 = up
        uint16_t* cp = C + (size_t)row * ldc + (n0 + (wn * TN + j) * 32) / 2 + feat_l;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float gt = acc[i][j][4 * g + e], up = acc[i][j + 1][4 * g + e];
            // the hardware reciprocal (1 ulp; the result is rounded to bf16 right after): an IEEE
            // division is eleven instructions, 64 of them per lane and tile
            v[e] = gt * __builtin_amdgcn_rcpf(1.0f + __expf(-gt)) * up;
          }
          uint2 w2;
          w2.x = pack_bf16(v[0], v[1]);
          w2.y = pack_bf16(v[2], v[3]);
          if (STAGED)
            *(uint2*)(sl + stage_off<NCH>((wm * TM + i) * 32 + tok_l,
                                          (wn * TN + j) * 16 + 8 * g + feat_l)) = w2;
          else
            *(uint2*)(cp + 8 * g) = w2;
        }
      }
    } else {
      float ss = 0.f;
      // the residual row: the output row, or the one the index names (compaction folded in)
      const size_t r_shift = (EPI == EPI_RESIDUAL && !STAGED && ra.r_rows != nullptr)
                                 ? ((size_t)ra.r_rows[row] - (size_t)row) * ldc : 0;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const size_t off = (size_t)row * ldc + n0 + (wn * TN + j) * 32 + feat_l;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = acc[i][j][4 * g + e];
          char* sp = STAGED ? sl + stage_off<NCH>((wm * TM + i) * 32 + tok_l,
                                                  (wn * TN + j) * 32 + 8 * g + feat_l) : nullptr;
          if (EPI == EPI_RESIDUAL) {
            // staged: the residual tile was copied into the same LDS slots beforehand
            const uint2 r2 = STAGED ? *(const uint2*)sp : *(const uint2*)(R + off + r_shift + 8 * g);
            v[0] += bf16_lo(r2.x); v[1] += bf16_hi(r2.x);
            v[2] += bf16_lo(r2.y); v[3] += bf16_hi(r2.y);
          }
          uint2 w2;
          w2.x = pack_bf16(v[0], v[1]);
          w2.y = pack_bf16(v[2], v[3]);
          if (STAGED) *(uint2*)sp = w2;
          else *(uint2*)(C + off + 8 * g) = w2;
          if (EPI == EPI_RESIDUAL) {
            const float a = bf16_lo(w2.x), b = bf16_hi(w2.x), c = bf16_lo(w2.y), e = bf16_hi(w2.y);
            ss += a * a + b * b + c * c + e * e;
          }
        }
      }
      if (EPI == EPI_RESIDUAL && ra.ssq_out != nullptr) {
        // rows past M left the loop above, so the partner lane (same token, other 4 features of
        // each group of 8) is active whenever this one is
        ss += __shfl_xor(ss, 32, 64);
        if (lane < 32) atomicAdd(ra.ssq_out + row, ssq_to_fixed(ss));
      }
    }
  }
}

// ---- workgroup -> tile.  Consecutive workgroup ids land on different XCDs (8 of them, each with
// its own L2), so ids are first regrouped per XCD, then walked in bands of group_m tile rows so
// that concurrently running tiles share A and W slabs in L2.
__device__ __forceinline__ void workgroup_tile(int pid, int tiles_m, int tiles_n, int group_m,
                                               int& tile_m, int& tile_n) {
  const int T = tiles_m * tiles_n;
  const int xcd = pid & 7, local = pid >> 3;
  const int per = (T + 7) >> 3;
  const int tall = (T & 7) == 0 ? 8 : (T & 7);
  const int np = xcd < tall ? xcd * per + local : tall * per + (xcd - tall) * (per - 1) + local;
  const int width = group_m * tiles_n;
  const int group = np / width;
  const int first_m = group * group_m;
  const int gsz = min(tiles_m - first_m, group_m);
  const int in_group = np - group * width;
  tile_m = first_m + in_group % gsz;
  tile_n = in_group / gsz;
}

// ---- staged output of a BM x BN tile held by NWAVES waves of TM x TN blocks (see stage_off):
// tile -> LDS in the MFMA layout's order, LDS -> global in whole rows.  `lds` is the kernel's
// dynamic LDS, free once every wave has left the K loop (the caller's copies have landed).
template <int TM, int TN, int EPI, int BM, int BN, int NWAVES>
__device__ __forceinline__ void staged_tile_out(floatx16_t (&acc)[TM][TN], uint16_t* __restrict__ C,
                                                const uint16_t* __restrict__ R, int M, int ldc, int m0,
                                                int n0, int wm, int wn, int wave, int lane,
                                                const EpiArgs& ra, const float* rs, char* lds) {
  // BNO = output columns of the tile, NCH = its 16-byte chunks per row
  constexpr int BNO = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
  constexpr int NCH = BNO / 8;
  static_assert((NCH & (NCH - 1)) == 0, "chunks per row must be a power of two");
  __syncthreads();                                  // every wave is done reading the stages
  if (EPI == EPI_RESIDUAL) {
    // the residual tile comes in the same way (whole rows, straight into LDS); a wave
    // instruction covers 64 / NCH rows
    constexpr int RPI = 64 / NCH, R_INSTR = BM / RPI / NWAVES;
#pragma unroll
    for (int q = 0; q < R_INSTR; ++q) {
      const int instr = wave * R_INSTR + q;
      const int rr = instr * RPI + lane / NCH;
      const int chunk = (lane % NCH) ^ (rr & (NCH - 1));
      int gr = m0 + rr;
      gr = gr < M ? gr : M - 1;
      if (ra.r_rows != nullptr) gr = ra.r_rows[gr];
      g2l16(R + (size_t)gr * ldc + n0 + chunk * 8, lds + instr * 1024);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  }
  gemm_epilogue<TM, TN, EPI, true, NCH>(acc, C, R, M, ldc, m0, n0, wm, wn, lane, ra, rs, lds);
  __syncthreads();
  uint16_t* obase;
  int old;
  const int32_t* orow = nullptr;                    // output row of tile row r, if not m0 + r
  if (EPI == EPI_QKV_ROPE64 || EPI == EPI_QKV_ROPE128) {
    const int dq = ra.d_model, kvd = ra.kv_dim > 0 ? ra.kv_dim : dq;
    const int region = n0 < dq ? 0 : n0 < dq + kvd ? 1 : 2;   // the tile lies inside q, k or v
    if (region == 2 && ra.v == nullptr) return;     // (the transposed copy went out with the epilogue)
    obase = (region == 0 ? ra.q : region == 1 ? ra.k : ra.v) +
            (n0 - (region == 0 ? 0 : region == 1 ? dq : dq + kvd));
    old = region == 0 ? dq : kvd;
    if (region == 1) orow = ra.k_row;
  } else {
    obase = C + (EPI == EPI_SWIGLU ? n0 / 2 : n0);
    old = ldc;
  }
  for (int idx = threadIdx.x; idx < BM * NCH; idx += NWAVES * 64) {
    const int r = idx / NCH, ch = idx % NCH;
    if (m0 + r < M) {
      const size_t dr = orow != nullptr ? (size_t)orow[m0 + r] : (size_t)(m0 + r);
      *(uint4*)(obase + dr * old + ch * 8) =
          *(const uint4*)(lds + r * (NCH * 16) + ((ch ^ (r & (NCH - 1))) << 4));
    }
  }
}

}  // namespace lz
