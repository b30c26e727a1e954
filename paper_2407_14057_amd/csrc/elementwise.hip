// Glue kernels of the decoder layer: plan, embedding, RMSNorm, rotary table, V transpose, final norm,
// LM head, and the weight repack used at model creation.  All bandwidth-bound; 16-byte
// vectors, one wave per row.
#include "common.h"

namespace lz {

// ------------------------------------------------------------------------------------------
// Per-stage row offsets.  Stage 0 is the full prompt; stage s+1 begins at the s-th pruning
// layer and keeps max(1, ceil(n * permille / 1000)) tokens of every sequence
// (Sec. 3.2: top-k percentile of the surviving tokens).  Counts do not depend on the data,
// so the whole table is known before the first layer runs.
// ------------------------------------------------------------------------------------------
// The caller sizes every buffer and launch from its host copy of the sequence lengths, so the
// tables must come from those same lengths: they arrive by value (kernel arguments, LENS_PER_LAUNCH
// at a time) in row 0 of cu_stage before plan_kernel runs.  The device copy of the offsets is only
// compared against them: any difference raises ST_BAD_CU, and the tables stay those of the host's
// lengths, inside the buffers it laid out.
__global__ void put_lens_kernel(LensChunk chunk, int offset, int count, int32_t* __restrict__ cu_stage) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) cu_stage[offset + i + 1] = chunk.n[i];
}

__global__ void plan_kernel(const int32_t* __restrict__ cu_dev, int n_single, int batch,
                            int expect_total, PlanArgs plan, int32_t* __restrict__ cu_stage,
                            int32_t* __restrict__ cu_aux, int32_t* __restrict__ cu_vt,
                            int32_t* __restrict__ status) {
  const int S = plan.n_stages + 1, W = batch + 1;
  __shared__ int bad;
  if (threadIdx.x == 0) {
    bad = 0;
    if (cu_dev != nullptr && (cu_dev[0] != 0 || cu_dev[batch] != expect_total)) bad = 1;
  }
  __syncthreads();
  for (int b = threadIdx.x; b < batch; b += blockDim.x) {
    int n = batch == 1 ? n_single : cu_stage[0 * W + b + 1];     // the host's length of sequence b
    if (n < 1) n = 1;
    if (cu_dev != nullptr && cu_dev[b + 1] - cu_dev[b] != n) bad = 1;   // (benign race: all write 1)
    cu_stage[0 * W + b + 1] = n;
    for (int s = 1; s < S; ++s) {
      long long k = ((long long)n * plan.permille[s - 1] + 999) / 1000;
      int kk = k < 1 ? 1 : (int)k;
      cu_aux[(s - 1) * W + b + 1] = n - kk;
      n = kk;
      cu_stage[s * W + b + 1] = n;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) *status = bad ? ST_BAD_CU : 0;
  // prefix sums over the batch, one stage per thread
  for (int s = threadIdx.x; s < S; s += blockDim.x) {
    int acc = 0, accv = 0;
    cu_stage[s * W] = 0;
    cu_vt[s * W] = 0;
    for (int b = 0; b < batch; ++b) {
      int n = cu_stage[s * W + b + 1];
      acc += n;
      accv += (n + 63) & ~63;
      cu_stage[s * W + b + 1] = acc;
      cu_vt[s * W + b + 1] = accv;
    }
    if (s >= 1) {
      int a = 0;
      cu_aux[(s - 1) * W] = 0;
      for (int b = 0; b < batch; ++b) {
        a += cu_aux[(s - 1) * W + b + 1];
        cu_aux[(s - 1) * W + b + 1] = a;
      }
    }
  }
}

hipError_t launch_plan(const int32_t* cu_dev, const int32_t* seqlens_host, int batch, int expect_total,
                       const PlanArgs& plan, int32_t* cu_stage, int32_t* cu_aux, int32_t* cu_vt,
                       int32_t* status, hipStream_t st) {
  if (batch > 1) {
    for (int off = 0; off < batch; off += LENS_PER_LAUNCH) {
      LensChunk chunk;
      const int count = batch - off < LENS_PER_LAUNCH ? batch - off : LENS_PER_LAUNCH;
      for (int i = 0; i < count; ++i) chunk.n[i] = seqlens_host[off + i];
      for (int i = count; i < LENS_PER_LAUNCH; ++i) chunk.n[i] = 0;
      hipLaunchKernelGGL(put_lens_kernel, dim3((count + 255) / 256), dim3(256), 0, st, chunk, off, count,
                         cu_stage);
    }
  }
  hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(64), 0, st, cu_dev, seqlens_host[0], batch, expect_total,
                     plan, cu_stage, cu_aux, cu_vt, status);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Rotary table: table[p][i] = (cos, sin)(p * theta^(-2i/hd)), angles formed in fp64.
// ------------------------------------------------------------------------------------------
__global__ void rope_table_kernel(float2* __restrict__ table, int n_pos, int half, double theta) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_pos * half) return;
  int p = idx / half, i = idx - p * half;
  double inv_freq = pow(theta, -(double)i / (double)half);
  double s, c;
  sincos((double)p * inv_freq, &s, &c);
  table[idx] = make_float2((float)c, (float)s);
}

hipError_t launch_rope_table(float2* table, int n_pos, int head_dim, float theta, hipStream_t st) {
  int half = head_dim / 2, total = n_pos * half;
  hipLaunchKernelGGL(rope_table_kernel, dim3((total + 255) / 256), dim3(256), 0, st, table, n_pos,
                     half, (double)theta);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Embedding gather (+ optional per-token scale) and position ids.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
embed_kernel(const uint4* __restrict__ embed, const int32_t* __restrict__ ids,
             const float* __restrict__ scale, const int32_t* __restrict__ cu, int batch, int total,
             int vec_per_row, int vocab, uint4* __restrict__ h, int32_t* __restrict__ pos,
             int32_t* __restrict__ status, unsigned long long* __restrict__ ssq) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + wave;
  if (row >= total) return;
  int id = ids[row];
  if (id < 0 || id >= vocab) {
    if (lane == 0) atomicOr(status, 1);
    id = id < 0 ? 0 : vocab - 1;
  }
  if (lane == 0) {
    int start = 0;
    if (cu != nullptr) {
      int lo = 0, hi = batch;                 // largest b with cu[b] <= row
      while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (cu[mid] <= row) lo = mid; else hi = mid;
      }
      start = cu[lo];
    }
    pos[row] = row - start;
  }
  const uint4* src = embed + (size_t)id * vec_per_row;
  uint4* dst = h + (size_t)row * vec_per_row;
  float ss = 0.f;                       // sum of squares of the row as stored (for the first RMSNorm)
  if (scale == nullptr) {
    for (int v = lane; v < vec_per_row; v += 64) {
      const uint4 x = src[v];
      dst[v] = x;
      float f[8];
      unpack8(x, f);
#pragma unroll
      for (int e = 0; e < 8; ++e) ss += f[e] * f[e];
    }
  } else {
    const float sc = scale[row];
    for (int v = lane; v < vec_per_row; v += 64) {
      float f[8];
      unpack8(src[v], f);
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] *= sc;
      const uint4 x = pack8(f);
      dst[v] = x;
      unpack8(x, f);
#pragma unroll
      for (int e = 0; e < 8; ++e) ss += f[e] * f[e];
    }
  }
  if (ssq != nullptr) {
    ss = wave_sum(ss);
    if (lane == 0) ssq[row] = ssq_to_fixed(ss);
  }
}

hipError_t launch_embed(const void* embed, const int32_t* ids, const float* scale, const int32_t* cu,
                        int batch, int total, int d, int vocab, void* h, int32_t* pos,
                        int32_t* status, hipStream_t st, unsigned long long* ssq) {
  hipLaunchKernelGGL(embed_kernel, dim3((total + 3) / 4), dim3(256), 0, st, (const uint4*)embed, ids,
                     scale, cu, batch, total, d / 8, vocab, (uint4*)h, pos, status, ssq);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// RMSNorm: one wave per row, the row stays in registers between the two passes.
// ------------------------------------------------------------------------------------------
template <int NV>
__global__ void __launch_bounds__(256)
rmsnorm_kernel(const uint4* __restrict__ h, const uint4* __restrict__ gain, uint4* __restrict__ x,
               int rows, int vec_per_row, float inv_d, float eps) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + wave;
  if (row >= rows) return;
  const uint4* src = h + (size_t)row * vec_per_row;
  uint4 reg[NV];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    int v = lane + 64 * i;
    if (v < vec_per_row) {
      reg[i] = src[v];
      float f[8];
      unpack8(reg[i], f);
#pragma unroll
      for (int e = 0; e < 8; ++e) ss += f[e] * f[e];
    }
  }
  ss = wave_sum(ss);
  const float r = rsqrtf(ss * inv_d + eps);
  uint4* dst = x + (size_t)row * vec_per_row;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    int v = lane + 64 * i;
    if (v < vec_per_row) {
      float f[8], g[8];
      unpack8(reg[i], f);
      unpack8(gain[v], g);
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] = f[e] * r * g[e];
      dst[v] = pack8(f);
    }
  }
}

hipError_t launch_rmsnorm(const void* h, const void* gain, void* x, int rows, int d, float eps,
                          hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  const int vpr = d / 8, nv = (vpr + 63) / 64;
  dim3 grid((rows + 3) / 4), block(256);
  const float inv_d = 1.0f / (float)d;
#define LZ_RMS(NV)                                                                              \
  hipLaunchKernelGGL(rmsnorm_kernel<NV>, grid, block, 0, st, (const uint4*)h, (const uint4*)gain, \
                     (uint4*)x, rows, vpr, inv_d, eps)
  if (nv <= 1) LZ_RMS(1);
  else if (nv <= 2) LZ_RMS(2);
  else if (nv <= 4) LZ_RMS(4);
  else if (nv <= 8) LZ_RMS(8);
  else if (nv <= 16) LZ_RMS(16);
  else if (nv <= 32) LZ_RMS(32);
  else return hipErrorInvalidValue;
#undef LZ_RMS
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Transposed copy of V for the attention kernel's second product: vt[h][dim][cu_vt[b] + token]
// (keys contiguous).  One workgroup = 64 tokens of one head, through an LDS tile.  The tail
// columns up to the next multiple of 64 are zeroed so that masked probabilities never meet a
// NaN.
// ------------------------------------------------------------------------------------------
template <int HD>
__global__ void __launch_bounds__(256)
v_transpose_kernel(const uint16_t* __restrict__ v, uint16_t* __restrict__ vt,
                   const int32_t* __restrict__ cu, const int32_t* __restrict__ cu_vt, int n_single,
                   int vt_ld, int n_heads) {
  constexpr int CH = HD / 8;            // 16-byte chunks per head row
  constexpr int LROW = HD + 2;          // padded LDS row (elements)
  __shared__ uint16_t tile[64 * LROW];
  const int b = blockIdx.z, head = blockIdx.y;
  int row0, n;
  seq_range(cu, b, n_single, row0, n);
  const int t0 = blockIdx.x * 64;
  if (t0 >= n) return;
  const int d = n_heads * HD;
  for (int idx = threadIdx.x; idx < 64 * CH; idx += 256) {
    const int t = idx / CH, c = idx % CH;
    uint4 val = make_uint4(0, 0, 0, 0);
    if (t0 + t < n) val = *(const uint4*)(v + (size_t)(row0 + t0 + t) * d + head * HD + c * 8);
    uint32_t* p = (uint32_t*)(tile + t * LROW + c * 8);   // LROW even: 4-byte aligned
    p[0] = val.x; p[1] = val.y; p[2] = val.z; p[3] = val.w;
  }
  __syncthreads();
  // thread takes (dim, group of 8 tokens)
  const size_t vt_base = (size_t)head * HD * vt_ld + (cu_vt ? cu_vt[b] : 0) + t0;
  for (int idx = threadIdx.x; idx < HD * 8; idx += 256) {
    const int j = idx & 7, dim = idx >> 3;
    uint16_t e[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) e[i] = tile[(j * 8 + i) * LROW + dim];
    uint4 o;
    o.x = e[0] | ((uint32_t)e[1] << 16); o.y = e[2] | ((uint32_t)e[3] << 16);
    o.z = e[4] | ((uint32_t)e[5] << 16); o.w = e[6] | ((uint32_t)e[7] << 16);
    *(uint4*)(vt + vt_base + (size_t)dim * vt_ld + j * 8) = o;
  }
}

hipError_t launch_v_transpose(const void* v, void* vt, const int32_t* cu, const int32_t* cu_vt,
                              int n_single, int batch, int max_rows, int vt_ld, int n_heads,
                              int head_dim, hipStream_t st) {
  if (max_rows <= 0) return hipSuccess;
  dim3 grid((max_rows + 63) / 64, n_heads, batch), block(256);
  if (head_dim == 128)
    hipLaunchKernelGGL(v_transpose_kernel<128>, grid, block, 0, st, (const uint16_t*)v, (uint16_t*)vt,
                       cu, cu_vt, n_single, vt_ld, n_heads);
  else if (head_dim == 64)
    hipLaunchKernelGGL(v_transpose_kernel<64>, grid, block, 0, st, (const uint16_t*)v, (uint16_t*)vt,
                       cu, cu_vt, n_single, vt_ld, n_heads);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

__global__ void __launch_bounds__(256)
vt_stage_setup_kernel(uint16_t* __restrict__ vt, int32_t* __restrict__ vt_col,
                      const int32_t* __restrict__ cu, const int32_t* __restrict__ cu_vt,
                      int n_single, int vt_ld, int n_feat) {
  const int b = blockIdx.y;
  int row0, n;
  seq_range(cu, b, n_single, row0, n);
  const int col0 = cu_vt ? cu_vt[b] : 0;
  const int pad = ((n + 63) & ~63) - n;
  const int f = blockIdx.x * 256 + threadIdx.x;
  if (f < n_feat) {
    uint16_t* p = vt + (size_t)f * vt_ld + col0 + n;
    for (int i = 0; i < pad; ++i) p[i] = 0;
  }
  if (vt_col != nullptr)
    for (int t = blockIdx.x * 256 + threadIdx.x; t < n; t += gridDim.x * 256)
      vt_col[row0 + t] = col0 + t;
}

hipError_t launch_vt_stage_setup(void* vt, int32_t* vt_col, const int32_t* cu, const int32_t* cu_vt,
                                 int n_single, int batch, int vt_ld, int n_feat, hipStream_t st) {
  hipLaunchKernelGGL(vt_stage_setup_kernel, dim3((n_feat + 255) / 256, batch), dim3(256), 0, st,
                     (uint16_t*)vt, vt_col, cu, cu_vt, n_single, vt_ld, n_feat);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Final RMSNorm of each sequence's last row -> fp32, then the LM-head GEMV.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
final_norm_kernel(const uint16_t* __restrict__ h, const int32_t* __restrict__ cu, int n_single,
                  const uint16_t* __restrict__ gain, float* __restrict__ xf, int d, float eps) {
  __shared__ float red[4];
  const int b = blockIdx.x;
  int row0, n;
  seq_range(cu, b, n_single, row0, n);
  const uint16_t* row = h + (size_t)(row0 + n - 1) * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) {
    float f = bf16_to_float(row[i]);
    ss += f * f;
  }
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  ss = red[0] + red[1] + red[2] + red[3];
  const float r = rsqrtf(ss / (float)d + eps);
  for (int i = threadIdx.x; i < d; i += 256)
    xf[(size_t)b * d + i] = bf16_to_float(row[i]) * r * bf16_to_float(gain[i]);
}

hipError_t launch_final_norm(const void* h, const int32_t* cu, int n_single, int batch,
                             const void* gain, float* xf, int d, float eps, hipStream_t st) {
  hipLaunchKernelGGL(final_norm_kernel, dim3(batch), dim3(256), 0, st, (const uint16_t*)h, cu,
                     n_single, (const uint16_t*)gain, xf, d, eps);
  return hipGetLastError();
}

// One wave per vocabulary row; the row's 16-byte vectors are read once and reused for
// every sequence of the batch.  Reads V*d*2 bytes: HBM-bound.
__global__ void __launch_bounds__(256)
lm_head_kernel(const float* __restrict__ xf, const uint4* __restrict__ w, float* __restrict__ logits,
               int batch, int d, int vocab) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int vpr = d / 8;
  for (int r = 0; r < 4; ++r) {
    const int row = (blockIdx.x * 4 + wave) * 4 + r;
    if (row >= vocab) return;
    const uint4* src = w + (size_t)row * vpr;
    for (int b = 0; b < batch; ++b) {
      const float* x = xf + (size_t)b * d;
      float acc = 0.f;
      for (int v = lane; v < vpr; v += 64) {
        float f[8];
        unpack8(src[v], f);
        const float4 x0 = *(const float4*)(x + v * 8), x1 = *(const float4*)(x + v * 8 + 4);
        acc += f[0] * x0.x + f[1] * x0.y + f[2] * x0.z + f[3] * x0.w + f[4] * x1.x + f[5] * x1.y +
               f[6] * x1.z + f[7] * x1.w;
      }
      acc = wave_sum(acc);
      if (lane == 0) logits[(size_t)b * vocab + row] = acc;
    }
  }
}

hipError_t launch_lm_head(const float* xf, const void* w_lm, float* logits, int batch, int d,
                          int vocab, hipStream_t st) {
  hipLaunchKernelGGL(lm_head_kernel, dim3((vocab + 15) / 16), dim3(256), 0, st, xf,
                     (const uint4*)w_lm, logits, batch, d, vocab);
  return hipGetLastError();
}

// Final norm and LM head in one launch.  Every workgroup first normalises the `batch` last rows
// itself (8 KB each, from the L2; the 500 or so workgroups all need them and a launch of its own
// for this costs more than the repetition) into LDS as fp32, then streams its 64 vocabulary rows:
// a wave takes four rows at a time, 16-byte loads of all four in flight before the first use
// (eight per lane), x from LDS.  Reads V*d*2 bytes once: HBM-bound.
constexpr int LMH_ROWS_PER_WAVE = 16, LMH_ROWS_PER_WG = 4 * LMH_ROWS_PER_WAVE;
template <int BATCH_MAX>
__global__ void __launch_bounds__(256)
lm_head_fused_kernel(const uint16_t* __restrict__ h, const int32_t* __restrict__ cu, int n_single,
                     const uint16_t* __restrict__ gain, const uint4* __restrict__ w,
                     float* __restrict__ logits, int batch, int d, int vocab, float eps) {
  extern __shared__ __attribute__((aligned(16))) float xs[];     // [batch][d]
  __shared__ float red[4];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  for (int b = 0; b < batch; ++b) {
    int row0, n;
    seq_range(cu, b, n_single, row0, n);
    const uint16_t* row = h + (size_t)(row0 + n - 1) * d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += 256) {
      const float f = bf16_to_float(row[i]);
      ss += f * f;
    }
    ss = wave_sum(ss);
    __syncthreads();                                   // (red is reused from the sequence before)
    if (lane == 0) red[wave] = ss;
    __syncthreads();
    ss = red[0] + red[1] + red[2] + red[3];
    const float r = rsqrtf(ss / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += 256)
      xs[(size_t)b * d + i] = bf16_to_float(row[i]) * r * bf16_to_float(gain[i]);
  }
  __syncthreads();
  const int vpr = d / 8;
  const int first = blockIdx.x * LMH_ROWS_PER_WG + wave * LMH_ROWS_PER_WAVE;
  for (int r0 = first; r0 < first + LMH_ROWS_PER_WAVE && r0 < vocab; r0 += 4) {
    float acc[4][BATCH_MAX];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int b = 0; b < BATCH_MAX; ++b) acc[r][b] = 0.f;
    const uint4* src[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) src[r] = w + (size_t)min(r0 + r, vocab - 1) * vpr;   // (rows past the end: repeated, not stored)
    for (int v = lane; v < vpr; v += 128) {
      uint4 wv[4][2];
      const int v1 = v + 64 < vpr ? v + 64 : v;
#pragma unroll
      for (int r = 0; r < 4; ++r) { wv[r][0] = src[r][v]; wv[r][1] = src[r][v1]; }
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        if (u == 1 && v + 64 >= vpr) break;
        const int vv = u == 0 ? v : v1;
#pragma unroll
        for (int b = 0; b < BATCH_MAX; ++b) {
          if (b >= batch) break;
          const float4 x0 = *(const float4*)(xs + (size_t)b * d + vv * 8);
          const float4 x1 = *(const float4*)(xs + (size_t)b * d + vv * 8 + 4);
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            float f[8];
            unpack8(wv[r][u], f);
            acc[r][b] += f[0] * x0.x + f[1] * x0.y + f[2] * x0.z + f[3] * x0.w + f[4] * x1.x + f[5] * x1.y +
                         f[6] * x1.z + f[7] * x1.w;
          }
        }
      }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int b = 0; b < BATCH_MAX; ++b) {
        if (b >= batch) break;
        const float t = wave_sum(acc[r][b]);
        if (lane == 0 && r0 + r < vocab) logits[(size_t)b * vocab + r0 + r] = t;
      }
  }
}

// logits[b] = rmsnorm(last row of sequence b) . W_lm^T; false if the shape does not fit this form
// (then the caller uses launch_final_norm + launch_lm_head).
bool lm_head_fused_fits(int batch, int d) {
  return batch >= 1 && batch <= 8 && d % 8 == 0 && (size_t)batch * d * 4 <= 128 * 1024;
}

hipError_t launch_lm_head_fused(const void* h, const int32_t* cu, int n_single, int batch, const void* gain,
                                const void* w_lm, float* logits, int d, int vocab, float eps, hipStream_t st) {
  if (!lm_head_fused_fits(batch, d)) return hipErrorInvalidValue;
  const size_t lds = (size_t)batch * d * 4;
  const dim3 grid((vocab + LMH_ROWS_PER_WG - 1) / LMH_ROWS_PER_WG), block(256);
#define LZ_LMH(BM)                                                                                 \
  do {                                                                                             \
    auto kern = lm_head_fused_kernel<BM>;                                                          \
    static bool attr_set = false;                                                                  \
    if (!attr_set) {                                                                               \
      hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                         128 * 1024);                                              \
      if (e != hipSuccess) return e;                                                               \
      attr_set = true;                                                                             \
    }                                                                                              \
    hipLaunchKernelGGL(kern, grid, block, lds, st, (const uint16_t*)h, cu, n_single,               \
                       (const uint16_t*)gain, (const uint4*)w_lm, logits, batch, d, vocab, eps);   \
  } while (0)
  if (batch == 1) LZ_LMH(1);
  else if (batch <= 4) LZ_LMH(4);
  else LZ_LMH(8);
#undef LZ_LMH
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Weight repack (model creation only).
// ------------------------------------------------------------------------------------------
__global__ void copy_rows_kernel(const uint16_t* __restrict__ src, uint16_t* __restrict__ dst,
                                 int rows, int cols, int src_ld, int dst_ld) {
  // dst[r][c] = c < cols ? src[r][c] : 0 for c < dst_ld
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t total = (size_t)rows * dst_ld;
  if (idx >= total) return;
  int r = (int)(idx / dst_ld), c = (int)(idx % dst_ld);
  dst[idx] = c < cols ? src[(size_t)r * src_ld + c] : (uint16_t)0;
}

hipError_t launch_copy_rows(const void* src, void* dst, int rows, int cols, int src_ld, int dst_ld,
                            hipStream_t st) {
  size_t total = (size_t)rows * dst_ld;
  hipLaunchKernelGGL(copy_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                     (const uint16_t*)src, (uint16_t*)dst, rows, cols, src_ld, dst_ld);
  return hipGetLastError();
}

// w[r][c] *= gain[c]: folds an RMSNorm gain into the projection that consumes the normalised row
// (exact when the gain is 1).
__global__ void scale_cols_kernel(uint16_t* __restrict__ w, const uint16_t* __restrict__ gain,
                                  size_t total, int cols) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  w[idx] = to_bf16(bf16_to_float(w[idx]) * bf16_to_float(gain[idx % cols]));
}

hipError_t launch_scale_cols(void* w, const void* gain, size_t rows, int cols, hipStream_t st) {
  const size_t total = rows * (size_t)cols;
  hipLaunchKernelGGL(scale_cols_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                     (uint16_t*)w, (const uint16_t*)gain, total, cols);
  return hipGetLastError();
}

__global__ void interleave_gate_up_kernel(const uint16_t* __restrict__ gate,
                                          const uint16_t* __restrict__ up,
                                          uint16_t* __restrict__ dst, int f, int f_pad, int d) {
  // dst row 64*j + i      = gate row 32*j + i   (i < 32)
  // dst row 64*j + 32 + i = up   row 32*j + i;  rows beyond f are zero
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t total = (size_t)2 * f_pad * d;
  if (idx >= total) return;
  int r = (int)(idx / d), c = (int)(idx % d);
  int j = r >> 6, i = r & 63;
  int srow = 32 * j + (i & 31);
  const uint16_t* src = (i < 32) ? gate : up;
  dst[idx] = srow < f ? src[(size_t)srow * d + c] : (uint16_t)0;
}

hipError_t launch_interleave_gate_up(const void* gate, const void* up, void* dst, int f, int f_pad,
                                     int d, hipStream_t st) {
  size_t total = (size_t)2 * f_pad * d;
  hipLaunchKernelGGL(interleave_gate_up_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                     st, (const uint16_t*)gate, (const uint16_t*)up, (uint16_t*)dst, f, f_pad, d);
  return hipGetLastError();
}

}  // namespace lz
