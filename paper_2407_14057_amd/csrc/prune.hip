// The pruning half of the path: Eq. 1 scoring, top-k percentile selection, compaction and
// Aux Cache write (Sec. 3.2).  Scoring and compaction are HBM-bound; selection works in LDS.
#include "common.h"

namespace lz {

// ------------------------------------------------------------------------------------------
// Scoring (Eq. 1) in three launches.
//   1. score_logits: z[h][j] = q_last[h] . k[j][h] / sqrt(hd) for every token j, plus each
//      workgroup's (max, sum exp) per head.  A wave streams whole token rows (all heads, 16-byte
//      chunks), two rows in flight; K is read exactly once.  Lane l owns chunks l + 64*i of the
//      row; one head is HD/8 consecutive chunks, so a head's dot product is a DPP reduction over
//      HD/8 adjacent lanes.  Tokens per workgroup (8..64) grow with the sequence so that short
//      sequences still fill the chip and long ones amortise the per-workgroup work.
//   2. score_stats: one workgroup per sequence folds the partials into (max_h, 1/Z_h), in a
//      fixed order (deterministic).
//   3. score_finish: s[j] = (1/H) sum_h exp(z[h][j] - max_h) / Z_h, heads added in order.
// ------------------------------------------------------------------------------------------
constexpr int SCORE_MAX_HEADS = 256;

__host__ __device__ inline int score_tok_per_wg(int max_rows) {
  return max_rows >= 65536 ? 64 : max_rows >= 16384 ? 32 : max_rows >= 6144 ? 16 : 8;
}

// Sum over groups of LPH (8 or 16) adjacent lanes with DPP moves (no LDS traffic); every lane
// of a group ends up with the group's sum.
template <int LPH>
__device__ __forceinline__ float group_sum(float v) {
  v += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0xB1, 0xf, 0xf, true));   // lane ^ 1
  v += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0x4E, 0xf, 0xf, true));   // lane ^ 2
  v += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0x141, 0xf, 0xf, true));  // mirror in 8
  if (LPH == 16)
    v += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0x140, 0xf, 0xf, true)); // mirror in 16
  return v;
}

template <int HD, int NV>   // NV = ceil(H*HD/8 / 64): chunks per lane
__global__ void __launch_bounds__(256)
score_logits_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                    float* __restrict__ z, float2* __restrict__ part,
                    const int32_t* __restrict__ cu, int n_single, int n_heads, int z_ld,
                    float scale, int tok) {
  constexpr int LPH = HD / 8;                   // lanes per head
  extern __shared__ float zs[];                 // [tok][n_heads + 1]
  const int zrow = n_heads + 1;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int b = blockIdx.y;
  int row0, n;
  seq_range(cu, b, n_single, row0, n);
  const int t0 = blockIdx.x * tok;
  if (t0 >= n) return;
  const int d = n_heads * HD, vpr = d / 8;
  const uint4* qrow = (const uint4*)(q + (size_t)(row0 + n - 1) * d);

  float qf[NV][8];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int v = lane + 64 * i;
    if (v < vpr) unpack8(qrow[v], qf[i]);
    else
#pragma unroll
      for (int e = 0; e < 8; ++e) qf[i][e] = 0.f;
  }

  const int tpw = tok >> 2;                      // tokens per wave, a multiple of 2
  for (int tl0 = wave * tpw; tl0 < (wave + 1) * tpw; tl0 += 2) {
    if (t0 + tl0 >= n) break;
    uint4 kv[2][NV];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      int t = t0 + tl0 + u;
      if (t >= n) t = n - 1;                     // clamp: result discarded below
      const uint4* krow = (const uint4*)(k + (size_t)(row0 + t) * d);
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int v = lane + 64 * i;
        kv[u][i] = (v < vpr) ? krow[v] : make_uint4(0, 0, 0, 0);
      }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        float kf[8];
        unpack8(kv[u][i], kf);
        float p = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) p += qf[i][e] * kf[e];
        p = group_sum<LPH>(p);
        const int head = (lane + 64 * i) / LPH;
        if ((lane % LPH) == 0 && head < n_heads) zs[(tl0 + u) * zrow + head] = p * scale;
      }
    }
  }
  __syncthreads();
  const int nt = min(tok, n - t0);
  // coalesced write of z[h][t0 .. t0+nt) and the workgroup's per-head partials
  for (int idx = threadIdx.x; idx < n_heads * tok; idx += 256) {
    const int h = idx / tok, t = idx % tok;
    if (t < nt) z[(size_t)h * z_ld + row0 + t0 + t] = zs[t * zrow + h];
  }
  for (int h = threadIdx.x; h < n_heads; h += 256) {
    float mx = -INFINITY;
    for (int t = 0; t < nt; ++t) mx = fmaxf(mx, zs[t * zrow + h]);
    float sum = 0.f;
    for (int t = 0; t < nt; ++t) sum += __expf(zs[t * zrow + h] - mx);
    part[((size_t)b * gridDim.x + blockIdx.x) * n_heads + h] = make_float2(mx, sum);
  }
}

__global__ void __launch_bounds__(256)
score_stats_kernel(const float2* __restrict__ part, float2* __restrict__ hstat,
                   const int32_t* __restrict__ cu, int n_single, int n_heads, int parts_per_seq,
                   int tok) {
  __shared__ float2 grp[256];
  const int b = blockIdx.x;
  int row0, n;
  seq_range(cu, b, n_single, row0, n);
  const int nparts = (n + tok - 1) / tok;
  const float2* p0 = part + (size_t)b * parts_per_seq * n_heads;
  for (int hb = 0; hb < n_heads; hb += 256) {           // heads in slabs of up to 256
    const int hcount = min(256, n_heads - hb);
    const int groups = max(1, 256 / hcount);
    const int g = threadIdx.x / hcount, hl = threadIdx.x % hcount;
    float mx = -INFINITY, sum = 0.f;
    if (g < groups) {
      // eight independent loads in flight per round: the fold is latency-bound otherwise
      for (int i0 = g; i0 < nparts; i0 += 8 * groups) {
        float2 pr[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int i = i0 + u * groups;
          pr[u] = i < nparts ? p0[(size_t)i * n_heads + hb + hl] : make_float2(-INFINITY, 0.f);
        }
        float nm = mx;
#pragma unroll
        for (int u = 0; u < 8; ++u) nm = fmaxf(nm, pr[u].x);
        float acc = sum * __expf(mx - nm);
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (pr[u].y > 0.f) acc += pr[u].y * __expf(pr[u].x - nm);
        sum = acc;
        mx = nm;
      }
    }
    grp[threadIdx.x] = make_float2(mx, sum);
    __syncthreads();
    if (threadIdx.x < hcount) {
      float M = -INFINITY;
      for (int gg = 0; gg < groups; ++gg) M = fmaxf(M, grp[gg * hcount + threadIdx.x].x);
      float Z = 0.f;
      for (int gg = 0; gg < groups; ++gg) {
        const float2 pr = grp[gg * hcount + threadIdx.x];
        if (pr.y > 0.f) Z += pr.y * __expf(pr.x - M);
      }
      hstat[(size_t)b * n_heads + hb + threadIdx.x] = make_float2(M, 1.0f / Z);
    }
    __syncthreads();
  }
}

template <bool BASE2>   // logits and reference points in the base-2 domain (attention kernel's)
__global__ void __launch_bounds__(256)
score_finish_kernel(const float* __restrict__ z, const float2* __restrict__ hstat,
                    float* __restrict__ s, const int32_t* __restrict__ cu, int n_single,
                    int n_heads, int z_ld, const int32_t* __restrict__ cu_z, bool padded) {
  __shared__ float2 hs[SCORE_MAX_HEADS];
  score_finish_block<BASE2>(z, hstat, s, cu, n_single, n_heads, z_ld, cu_z, padded, blockIdx.y,
                            blockIdx.x * 256, hs);
}

// scratch layout: z[H][total_rows] fp32 | hstat[batch][H] float2 | partials (upper bound)
size_t score_scratch_bytes(int total_rows, int batch, int n_heads) {
  // rows padded per sequence to a multiple of 64 (the layout the attention kernel writes)
  size_t zb = (size_t)n_heads * ((size_t)total_rows + 64 * (size_t)batch) * sizeof(float);
  zb = (zb + 255) & ~(size_t)255;
  size_t hb = ((size_t)batch * n_heads * sizeof(float2) + 255) & ~(size_t)255;
  size_t parts = (size_t)batch * ((size_t)(total_rows + 7) / 8 + 1);
  return zb + hb + parts * n_heads * sizeof(float2) + 256;
}

hipError_t launch_score(const void* q, const void* k, float* s, void* scratch, const int32_t* cu,
                        int n_single, int batch, int total_rows, int max_rows, int n_heads,
                        int head_dim, hipStream_t st) {
  if (max_rows <= 0) return hipSuccess;
  if (n_heads > SCORE_MAX_HEADS) return hipErrorInvalidValue;
  float* z = (float*)scratch;
  size_t zb = (size_t)n_heads * total_rows * sizeof(float);
  zb = (zb + 255) & ~(size_t)255;
  float2* hstat = (float2*)((char*)scratch + zb);
  size_t hb = ((size_t)batch * n_heads * sizeof(float2) + 255) & ~(size_t)255;
  float2* part = (float2*)((char*)scratch + zb + hb);
  const int tok = score_tok_per_wg(max_rows);
  const int parts_per_seq = (max_rows + tok - 1) / tok;
  const int vpr = n_heads * head_dim / 8, nv = (vpr + 63) / 64;
  const float scale = 1.0f / sqrtf((float)head_dim);
  const size_t lds = (size_t)tok * (n_heads + 1) * sizeof(float);
  dim3 grid(parts_per_seq, batch), block(256);
#define LZ_SCORE(HD, NV)                                                                        \
  hipLaunchKernelGGL((score_logits_kernel<HD, NV>), grid, block, lds, st, (const uint16_t*)q,    \
                     (const uint16_t*)k, z, part, cu, n_single, n_heads, total_rows, scale, tok)
  if (head_dim == 128) {
    if (nv <= 1) LZ_SCORE(128, 1);
    else if (nv <= 2) LZ_SCORE(128, 2);
    else if (nv <= 4) LZ_SCORE(128, 4);
    else if (nv <= 8) LZ_SCORE(128, 8);
    else if (nv <= 16) LZ_SCORE(128, 16);
    else return hipErrorInvalidValue;
  } else if (head_dim == 64) {
    if (nv <= 1) LZ_SCORE(64, 1);
    else if (nv <= 2) LZ_SCORE(64, 2);
    else if (nv <= 4) LZ_SCORE(64, 4);
    else if (nv <= 8) LZ_SCORE(64, 8);
    else if (nv <= 16) LZ_SCORE(64, 16);
    else return hipErrorInvalidValue;
  } else {
    return hipErrorInvalidValue;
  }
#undef LZ_SCORE
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(score_stats_kernel, dim3(batch), dim3(256), 0, st, part, hstat, cu, n_single,
                     n_heads, parts_per_seq, tok);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(score_finish_kernel<false>, dim3((max_rows + 255) / 256, batch), dim3(256), 0,
                     st, z, hstat, s, cu, n_single, n_heads, total_rows, nullptr, false);
  return hipGetLastError();
}

float* score_z(void* scratch) { return (float*)scratch; }

// The attention kernel writes logits in the padded layout of the Vt buffer: row length z_ld
// (a multiple of 64, at least the padded token count), sequence b at offset cu_z[b].
void* score_zstat(void* scratch, int z_ld, int n_heads) {
  size_t zb = (size_t)n_heads * z_ld * sizeof(float);
  zb = (zb + 255) & ~(size_t)255;
  return (char*)scratch + zb;
}

hipError_t launch_score_finish(float* s, void* scratch, const int32_t* cu, const int32_t* cu_z,
                               int n_single, int batch, int z_ld, int max_rows, int n_heads,
                               hipStream_t st) {
  if (max_rows <= 0) return hipSuccess;
  if (n_heads > SCORE_MAX_HEADS) return hipErrorInvalidValue;
  hipLaunchKernelGGL(score_finish_kernel<true>, dim3((max_rows + 255) / 256, batch), dim3(256), 0,
                     st, score_z(scratch), (const float2*)score_zstat(scratch, z_ld, n_heads), s,
                     cu, n_single, n_heads, z_ld, cu_z, true);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Selection: keep the last token and the k-1 best of the others (higher score, then lower
// index).  One 1024-thread workgroup per sequence.  Scores become order-preserving 32-bit
// keys held in LDS; an MSB-first radix select (4 passes of 8 bits, LDS histogram, one wave
// scanning the 256 bins) finds the threshold key and how many of its duplicates to take;
// a final ordered pass emits kept and pruned row indices, ranks coming from wave ballots
// and a per-wave prefix.
// ------------------------------------------------------------------------------------------
constexpr int SEL_THREADS = 1024;
constexpr int SEL_WAVES = SEL_THREADS / 64;
constexpr int SEL_LDS_KEYS = 15360;   // 60 KB of keys; longer sequences re-read global memory

__device__ __forceinline__ uint32_t score_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// exclusive rank of this thread among threads with flag set, and the block total.
// Must be called by all threads.  wsum: LDS [SEL_WAVES].
__device__ __forceinline__ int block_rank(bool flag, int* wsum, int& total) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const unsigned long long bal = __ballot(flag);
  const int below = __popcll(bal & ((1ull << lane) - 1ull));
  if (lane == 0) wsum[wave] = __popcll(bal);
  __syncthreads();
  int pre = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < SEL_WAVES; ++w) {
    const int c = wsum[w];
    if (w < wave) pre += c;
    tot += c;
  }
  __syncthreads();
  total = tot;
  return pre + below;
}

// The key of rank `need` (1-based, descending) among candidates 0..ncand-1 and how many of its
// duplicates belong to the top `need`: T = that key, need_eq = duplicates to take (in index
// order).  need <= 0: nothing qualifies (T = max key, need_eq = 0); need >= ncand: everything.
// MSB-first radix select, 4 passes of 8 bits.  Called by every thread of the workgroup;
// hist: LDS int[256], sel_bin / sel_need: LDS ints.
template <class KeyAt>
__device__ __forceinline__ void select_threshold(KeyAt key_at, int ncand, int m, int need, int* hist,
                                                 int* sel_bin, int* sel_need, uint32_t& T,
                                                 int& need_eq) {
  if (need <= 0) {
    T = 0xffffffffu; need_eq = 0;
  } else if (need >= ncand) {
    T = 0u; need_eq = m;
  } else {
    uint32_t prefix = 0u, mask = 0u;
    for (int shift = 24; shift >= 0; shift -= 8) {
      for (int i = threadIdx.x; i < 256; i += SEL_THREADS) hist[i] = 0;
      __syncthreads();
      for (int i = threadIdx.x; i < ncand; i += SEL_THREADS) {
        const uint32_t key = key_at(i);
        if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
      }
      __syncthreads();
      if (threadIdx.x < 64) {
        // lane L owns bins 255-4L .. 252-4L (descending); scan from the top bin down
        const int lane = threadIdx.x;
        const int top = 255 - 4 * lane;
        const int c0 = hist[top], c1 = hist[top - 1], c2 = hist[top - 2], c3 = hist[top - 3];
        const int local = c0 + c1 + c2 + c3;
        int incl = local;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
          const int t = __shfl_up(incl, o, 64);
          if (lane >= o) incl += t;
        }
        const int excl = incl - local;
        if (excl < need && need <= incl) {
          int acc = excl, bin = top, cnt = c0;
          if (acc + cnt < need) { acc += cnt; bin = top - 1; cnt = c1;
            if (acc + cnt < need) { acc += cnt; bin = top - 2; cnt = c2;
              if (acc + cnt < need) { acc += cnt; bin = top - 3; } } }
          *sel_bin = bin;
          *sel_need = need - acc;              // rank inside the chosen bin, >= 1
        }
      }
      __syncthreads();
      prefix |= ((uint32_t)*sel_bin) << shift;
      mask |= 255u << shift;
      need = *sel_need;
      __syncthreads();
    }
    T = prefix;
    need_eq = need;
  }
}

__global__ void __launch_bounds__(SEL_THREADS)
select_kernel(const float* __restrict__ s, const int32_t* __restrict__ cu_prev,
              const int32_t* __restrict__ cu_new, int m_single, int k_single,
              int32_t* __restrict__ keep_idx, int32_t* __restrict__ prune_idx) {
  __shared__ uint32_t keys[SEL_LDS_KEYS];
  __shared__ int hist[256];
  __shared__ int wsum[SEL_WAVES];
  __shared__ int sel_bin, sel_need;
  const int b = blockIdx.x;
  int r0, m, k0, k;
  seq_range(cu_prev, b, m_single, r0, m);
  seq_range(cu_new, b, k_single, k0, k);
  int32_t* keep_out = keep_idx + k0;
  int32_t* prune_out = prune_idx + (r0 - k0);
  const float* sv = s + r0;
  const bool in_lds = m <= SEL_LDS_KEYS;
  const int ncand = m - 1;                       // the last token is not a candidate

  if (in_lds) {
    for (int i = threadIdx.x; i < m; i += SEL_THREADS) keys[i] = score_key(sv[i]);
    __syncthreads();
  }
#define key_at(i) (in_lds ? keys[(i)] : score_key(sv[(i)]))

  uint32_t T;
  int need_eq;
  select_threshold([&](int i) { return key_at(i); }, ncand, m, k - 1, hist, &sel_bin, &sel_need, T, need_eq);

  // ordered emission
  int run_eq = 0, run_keep = 0;
  for (int base = 0; base < m; base += SEL_THREADS) {
    const int i = base + threadIdx.x;
    const bool valid = i < m;
    const bool last = valid && (i == m - 1);
    const uint32_t key = (valid && !last) ? key_at(i) : 0u;
    const bool gt = valid && !last && key > T;
    const bool eq = valid && !last && key == T;
    int tot_eq, tot_keep;
    const int eq_rank = run_eq + block_rank(eq, wsum, tot_eq);
    const bool keep = last || gt || (eq && eq_rank < need_eq);
    const int keep_rank = run_keep + block_rank(keep, wsum, tot_keep);
    if (valid) {
      if (keep) keep_out[keep_rank] = r0 + i;
      else prune_out[i - keep_rank] = r0 + i;
    }
    run_eq += tot_eq;
    run_keep += tot_keep;
  }
#undef key_at
}

hipError_t launch_select(const float* s, const int32_t* cu_prev, const int32_t* cu_new,
                         int m_single, int k_single, int batch, int32_t* keep_idx,
                         int32_t* prune_idx, hipStream_t st) {
  hipLaunchKernelGGL(select_kernel, dim3(batch), dim3(SEL_THREADS), 0, st, s, cu_prev, cu_new,
                     m_single, k_single, keep_idx, prune_idx);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Decoding, one pruning layer of one generation step (Sec. 3.2, "Aux Cache").  Everything is
// indexed by original position.  The same top-k rule as above picks k of the tokens selected
// at the layer below (member_prev; null = all n_tot tokens), by this step's scores of that
// layer; the new token (position n_tot-1) is forced.  Then every position is classified:
//   selected, K,V present at this layer        -> read from the KV cache, nothing to do
//   selected, no K,V                            -> runs the layer: gets the next row (ascending
//        position); its input is row live_row[] of the states carried out of the layer below in
//        this step, or else this layer's Aux Cache entry (src_row = -1)
//   not selected, but carrying a state          -> the state is parked in this layer's Aux Cache
// Outputs: member bytes and 64-bit words (the attention kernel's key mask), the row lists, the
// updated has_kv / has_aux / live_row tables, counts = {rows, parked, selected}.
// One 1024-thread workgroup.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(SEL_THREADS)
gen_stage_kernel(const float* __restrict__ s, const uint8_t* __restrict__ member_prev, int m, int k,
                 uint8_t* __restrict__ member, unsigned long long* __restrict__ member_bits,
                 uint8_t* __restrict__ has_kv, uint8_t* __restrict__ has_aux,
                 int32_t* __restrict__ live_row, int32_t* __restrict__ run_pos,
                 int32_t* __restrict__ src_row, int32_t* __restrict__ park_src,
                 int32_t* __restrict__ park_pos, int32_t* __restrict__ counts,
                 int32_t* __restrict__ status) {
  __shared__ uint32_t keys[SEL_LDS_KEYS];
  __shared__ int hist[256];
  __shared__ int wsum[SEL_WAVES];
  __shared__ int sel_bin, sel_need;
  const bool in_lds = m <= SEL_LDS_KEYS;
  const int ncand = m - 1;
  // tokens outside the candidate set get key 0, below every real score's key (scores are >= 0,
  // so their keys have the top bit set)
  auto make_key = [&](int i) -> uint32_t {
    return (member_prev != nullptr && member_prev[i] == 0) ? 0u : score_key(s[i]);
  };
  if (in_lds) {
    for (int i = threadIdx.x; i < m; i += SEL_THREADS) keys[i] = make_key(i);
    __syncthreads();
  }
  auto key_at = [&](int i) -> uint32_t { return in_lds ? keys[i] : make_key(i); };
  uint32_t T;
  int need_eq;
  select_threshold(key_at, ncand, m, k - 1, hist, &sel_bin, &sel_need, T, need_eq);

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int run_eq = 0, run_rows = 0, run_park = 0, run_sel = 0;
  for (int base = 0; base < m; base += SEL_THREADS) {
    const int i = base + threadIdx.x;
    const bool valid = i < m;
    const bool last = valid && (i == m - 1);
    const uint32_t key = (valid && !last) ? key_at(i) : 0u;
    const bool gt = valid && !last && key > T;
    const bool eq = valid && !last && key == T;
    int tot_eq, tot_rows, tot_park;
    const int eq_rank = run_eq + block_rank(eq, wsum, tot_eq);
    const bool sel = last || gt || (eq && eq_rank < need_eq);
    const bool kv = valid && has_kv[i] != 0;
    const int lr = valid ? live_row[i] : -1;
    const bool runs = sel && !kv;
    const bool park = valid && !sel && lr >= 0 && !kv;
    const int row = run_rows + block_rank(runs, wsum, tot_rows);
    const int pr = run_park + block_rank(park, wsum, tot_park);
    const unsigned long long word = __ballot(sel);
    if (valid) {
      member[i] = sel ? 1 : 0;
      if (runs) {
        run_pos[row] = i;
        src_row[row] = lr;
        has_kv[i] = 1;
        if (lr < 0 && has_aux[i] == 0) atomicOr(status, ST_NO_STATE);
      }
      live_row[i] = runs ? row : -1;
      if (park) {
        park_src[pr] = lr;
        park_pos[pr] = i;
        has_aux[i] = 1;
      }
    }
    if (lane == 0 && base + wave * 64 < m) member_bits[(base >> 6) + wave] = word;
    run_eq += tot_eq;
    run_rows += tot_rows;
    run_park += tot_park;
    run_sel += __popcll(word);          // per wave; summed below
  }
  // selected count: add the waves' partial sums
  if (lane == 0) wsum[wave] = run_sel;
  __syncthreads();
  if (threadIdx.x == 0) {
    int tot = 0;
    for (int w = 0; w < SEL_WAVES; ++w) tot += wsum[w];
    counts[0] = run_rows;
    counts[1] = run_park;
    counts[2] = tot;
  }
}

hipError_t launch_gen_stage(const float* s, const uint8_t* member_prev, int n_tot, int k,
                            uint8_t* member, unsigned long long* member_bits, uint8_t* has_kv,
                            uint8_t* has_aux, int32_t* live_row, int32_t* run_pos,
                            int32_t* src_row, int32_t* park_src, int32_t* park_pos,
                            int32_t* counts, int32_t* status, hipStream_t st) {
  hipLaunchKernelGGL(gen_stage_kernel, dim3(1), dim3(SEL_THREADS), 0, st, s, member_prev, n_tot, k,
                     member, member_bits, has_kv, has_aux, live_row, run_pos, src_row, park_src,
                     park_pos, counts, status);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Compaction + Aux Cache write: every input row is read once and written once, either to
// the compacted hidden states or to the Aux Cache of this pruning layer.  One wave per row.
// h_out == nullptr: the kept rows are read (for their sums of squares, which then go to ssq at the
// row's OLD index) but not copied: the caller's next projections read them through keep_idx.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
gather_kernel(const uint4* __restrict__ h, const int32_t* __restrict__ pos,
              const int32_t* __restrict__ keep_idx, int n_keep,
              const int32_t* __restrict__ prune_idx, int n_prune, uint4* __restrict__ h_out,
              int32_t* __restrict__ pos_out, uint4* __restrict__ aux_h,
              int32_t* __restrict__ aux_pos, int vpr, unsigned long long* __restrict__ ssq) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + wave;
  if (r >= n_keep + n_prune) return;
  int src_row;
  uint4* dst;
  if (r < n_keep) {
    src_row = keep_idx[r];
    if (lane == 0) pos_out[r] = pos[src_row];
    dst = h_out != nullptr ? h_out + (size_t)r * vpr : nullptr;
  } else {
    const int ra = r - n_keep;
    src_row = prune_idx[ra];
    dst = aux_h + (size_t)ra * vpr;
    if (lane == 0) aux_pos[ra] = pos[src_row];
  }
  const uint4* src = h + (size_t)src_row * vpr;
  const bool want_ssq = ssq != nullptr && r < n_keep;   // kept rows feed the next RMSNorm
  float ss = 0.f;
  int v = lane;
  for (; v + 64 * 7 < vpr; v += 64 * 8) {
    uint4 t[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = src[v + 64 * i];
    if (dst != nullptr) {
#pragma unroll
      for (int i = 0; i < 8; ++i) dst[v + 64 * i] = t[i];
    }
    if (want_ssq) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float f[8];
        unpack8(t[i], f);
#pragma unroll
        for (int e = 0; e < 8; ++e) ss += f[e] * f[e];
      }
    }
  }
  for (; v < vpr; v += 64) {
    const uint4 x = src[v];
    if (dst != nullptr) dst[v] = x;
    if (want_ssq) {
      float f[8];
      unpack8(x, f);
#pragma unroll
      for (int e = 0; e < 8; ++e) ss += f[e] * f[e];
    }
  }
  if (want_ssq) {
    ss = wave_sum(ss);
    if (lane == 0) ssq[h_out != nullptr ? r : src_row] = ssq_to_fixed(ss);
  }
}

hipError_t launch_gather(const void* h, const int32_t* pos, const int32_t* keep_idx, int n_keep,
                         const int32_t* prune_idx, int n_prune, void* h_out, int32_t* pos_out,
                         void* aux_h, int32_t* aux_pos, int d, hipStream_t st,
                         unsigned long long* ssq) {
  const int rows = n_keep + n_prune;
  if (rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(gather_kernel, dim3((rows + 3) / 4), dim3(256), 0, st, (const uint4*)h, pos,
                     keep_idx, n_keep, prune_idx, n_prune, (uint4*)h_out, pos_out, (uint4*)aux_h,
                     aux_pos, d / 8, ssq);
  return hipGetLastError();
}

}  // namespace lz
