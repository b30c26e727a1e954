// Shared device helpers and the host-side launch interface of the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lz {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx2_t __attribute__((ext_vector_type(2)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));

constexpr int WAVE = 64;

// ---- bf16 <-> fp32 (round to nearest even through v_cvt_pk_bf16_f32) -------------------
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  floatx2_t f = {lo, hi};
  bf16x2_t h = __builtin_convertvector(f, bf16x2_t);
  return *reinterpret_cast<uint32_t*>(&h);
}
__device__ __forceinline__ uint16_t to_bf16(float x) { return (uint16_t)(pack_bf16(x, 0.f) & 0xffffu); }
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_float(uint16_t u) { return __uint_as_float(((uint32_t)u) << 16); }

// 8 bf16 (one 16-byte vector) <-> 8 floats
__device__ __forceinline__ void unpack8(const uint4& v, float* f) {
  f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x); f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
  f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z); f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
}
__device__ __forceinline__ uint4 pack8(const float* f) {
  uint4 v;
  v.x = pack_bf16(f[0], f[1]); v.y = pack_bf16(f[2], f[3]);
  v.z = pack_bf16(f[4], f[5]); v.w = pack_bf16(f[6], f[7]);
  return v;
}

// ---- wave-level reductions (64 lanes) ---------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// ---- LDS tiles filled straight from global memory ---------------------------------------
// The gfx950 LDS is 64 banks x 4 bytes: a 16-byte-per-lane read is served 16 lanes at a
// time, and those 16 lanes must touch 16 different 16-byte units of the 256-byte bank line.
// MFMA operand reads have consecutive lanes on consecutive rows at one logical chunk, so
// chunk c of row r is stored at slot c ^ swz(r), with swz chosen so that 16 consecutive rows
// spread over all 16 units:
//   128-byte rows (2 per bank line): swz64(r) = (r >> 1) & 7
//    64-byte rows (4 per bank line): swz32(r) = (r >> 2) & 3
//   256-byte rows (1 per bank line): swz128(r) = r & 15
// global_load_lds writes lane i of a wave instruction to LDS base + 16*i, so the permutation
// is applied to the global address each lane fetches.
__device__ __forceinline__ int swz64(int row) { return (row >> 1) & 7; }
__device__ __forceinline__ int swz32(int row) { return (row >> 2) & 3; }
__device__ __forceinline__ int swz128(int row) { return row & 15; }

__device__ __forceinline__ void g2l16(const void* gsrc, void* lds_wave_base) {
  __builtin_amdgcn_global_load_lds(
      (const __attribute__((address_space(1))) void*)gsrc,
      (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}

// Row range of sequence b: from the offsets cu[batch+1], or [0, n_single) when cu is null
// (single-sequence calls need no device-side table).
__device__ __forceinline__ void seq_range(const int32_t* cu, int b, int n_single, int& row0, int& n) {
  if (cu != nullptr) { row0 = cu[b]; n = cu[b + 1] - row0; }
  else { row0 = 0; n = n_single; }
}

// Eq. 1 for `threads` consecutive tokens of sequence b starting at t0: s_j = (1/H) sum_h
// exp(z[h][j] - ref_h) / sum_h, heads added in order.  hs: n_heads float2 of LDS.  BASE2: logits and
// reference points in the base-2 domain (the attention kernel's).  padded: z rows are laid out
// like the Vt buffer (sequence b at cu_z[b]) instead of packed.
template <bool BASE2>
__device__ __forceinline__ void score_finish_block(const float* __restrict__ z,
                                                   const float2* __restrict__ hstat,
                                                   float* __restrict__ s, const int32_t* cu,
                                                   int n_single, int n_heads, int z_ld,
                                                   const int32_t* cu_z, bool padded, int b, int t0,
                                                   float2* hs) {
  int row0, n;
  seq_range(cu, b, n_single, row0, n);
  if (t0 >= n) return;
  for (int h = threadIdx.x; h < n_heads; h += blockDim.x) hs[h] = hstat[(size_t)b * n_heads + h];
  __syncthreads();
  const int t = t0 + threadIdx.x;
  if (t < n) {
    float acc = 0.f;
    const int zoff = padded ? (cu_z ? cu_z[b] : 0) : row0;   // where this sequence's logits start
    for (int h = 0; h < n_heads; ++h) {
      const float dz = z[(size_t)h * z_ld + zoff + t] - hs[h].x;
      acc += (BASE2 ? __builtin_amdgcn_exp2f(dz) : __expf(dz)) * hs[h].y;
    }
    s[row0 + t] = acc / (float)n_heads;
  }
}

// ---- launch interface (host) ------------------------------------------------------------
// EPI_QKV_ROPE is the caller-facing value; the kernel is instantiated per head size.
enum GemmEpilogue { EPI_STORE = 0, EPI_RESIDUAL = 1, EPI_SWIGLU = 2, EPI_QKV_ROPE = 3,
                    EPI_QKV_ROPE64 = 4, EPI_QKV_ROPE128 = 5 };

// Extra operands of the fused QKV + rotary epilogue: q, k, v are [rows, d_model] bf16,
// table is float2 [positions, head_dim/2] = (cos, sin), pos the original position of each row.
struct EpiArgs {
  // EPI_QKV_ROPE: rotary table and the three destinations
  const int32_t* pos;
  const float2* table;
  uint16_t* q;
  uint16_t* k;
  uint16_t* v;
  int d_model, head_dim;
  int kv_dim;                        // width of the k and v parts (K,V heads x head_dim); 0 = d_model
  // optional transposed copy of V for the attention kernel: vt[H*hd][vt_ld], token `row` in column
  // vt_col[row] (row itself when vt_col is null); vt == nullptr: not written
  uint16_t* vt;
  int vt_ld;
  const int32_t* vt_col;
  // caches indexed by something other than the GEMM's row (decoding: by original position):
  // token `row` writes its K to row k_row[row] (row itself when null); v == nullptr: the row-major
  // V is not written at all (only the transposed copy)
  const int32_t* k_row;
  // RMSNorm folded into the projections (gains are folded into the weights when the model is
  // made).  ssq_in: per token row, the sum of squares of the A operand's row as 2^-32 fixed point;
  // the epilogue multiplies row t of C by rsqrt(ssq_in[t] * ssq_mul + eps), ssq_mul = 2^-32 / K.
  // ssq_out: EPI_RESIDUAL adds the sum of squares of the (rounded) values it writes, one integer
  // atomic per wave and row -- integer addition commutes, so the total does not depend on the
  // order the waves arrive in.  ssq_clear: rows of this tile are zeroed there by the workgroups of
  // the first tile column (the buffer the next residual GEMM accumulates into).
  const unsigned long long* ssq_in;
  float ssq_mul, eps;
  unsigned long long* ssq_out;
  unsigned long long* ssq_clear;
  // Row indirection (compaction folded into the operand loads, Sec. 3.2's gather): row t of the A
  // operand, and of ssq_in, is row a_rows[t] of the buffers passed (rope epilogue's GEMMs); row
  // t of the residual R is row r_rows[t] (residual epilogue; C is then another buffer than R).
  // Null: the identity.
  const int32_t* a_rows;
  const int32_t* r_rows;
  // Side job for workgroups past the last tile (independent of the GEMM; it rides in this launch
  // because a launch of its own would cost more than the work): Eq. 1 from the logits the
  // attention kernel left, see score_finish_block.  sf_z == nullptr: none.
  const float* sf_z;
  const float2* sf_stat;
  float* sf_s;
  const int32_t* sf_cu;
  const int32_t* sf_cu_z;
  int sf_n_single, sf_heads, sf_z_ld, sf_max_rows, sf_batch;
  int sf_blocks_per_seq;             // filled in by the launcher (depends on the workgroup size)
  int stage_out;                     // filled in by the launcher: tile goes out through LDS (see gemm.hip)
  // the caller keeps the ticket counters at the end of the GEMM workspace zeroed
  // (launch_gemm_counters_clear once before the first use): M <= 32 may take the skinny kernel
  int skinny;
  // the caller keeps the flags of the persistent stream-K kernel (also at the end of the GEMM
  // workspace) zeroed likewise: launches whose tile count leaves the last round of the chip partly
  // idle may take that kernel
  int psk_ready;
  // filled in by the launcher: workgroups that walk the tiles of the ping-pong kernel's SiLU*mul
  // form, and their ticket counters (inside the flag area above; null: one workgroup per tile)
  int pp_walkers;
  unsigned* walk_tickets;
  // the W argument is in the weight-streaming kernel's own layout (launch_pack_stream); only that
  // kernel can read it, so the launch fails where another kernel would be chosen
  int w_packed;
  // the same weight in that layout, if the caller has one: used (instead of W) whenever the
  // weight-streaming kernel is chosen
  const void* w_stream;
  // W is stored K-step-major: [K / 64][N][64], each 64-element step of all rows contiguous (a
  // tile's W slab of one step is one contiguous run).  Filled in by the launcher: bytes from one
  // K step of a row to the next (128 for the row-major form).
  int w_blocked;
  unsigned long long w_step_bytes;
};
constexpr float SSQ_FIX = 4294967296.0f;      // 2^32
__device__ __forceinline__ unsigned long long ssq_to_fixed(float ss) {
  return (unsigned long long)(fminf(ss, 1.0e9f) * SSQ_FIX);
}

// records a failing HIP call for lazyllm_last_hip_error() (this thread)
void set_last_hip_error(int e);

// sk_ws: optional scratch of gemm_workspace_bytes() for the stream-K variant (fp32 partial tiles).
size_t gemm_workspace_bytes();
hipError_t launch_gemm(const void* A, const void* W, void* C, const void* R, int M, int N, int K,
                       int lda, int ldw, int ldc, int epilogue, hipStream_t st,
                       const EpiArgs* rope = nullptr, void* sk_ws = nullptr, size_t sk_ws_bytes = 0);

// The 256x256 tile on four waves of 128x128, one per SIMD (gemm_w4.hip); N % 256 == 0.
hipError_t launch_gemm_w4(const void* A, const void* W, void* C, const void* R, int M, int N, int K,
                          int lda, int ldw, int ldc, int epi, int group_m, const EpiArgs& ra,
                          hipStream_t st);
hipError_t launch_gemm_counters_clear(void* sk_ws, hipStream_t st);
// ORs ST_EXCHANGE into *status if a GEMM since the last clear gave up on an exchange of partial
// tiles between its workgroups (a flag that never came, or came from another XCD): its output,
// and everything computed from it, is then not to be used.
hipError_t launch_gemm_exchange_check(const void* sk_ws, int32_t* status, hipStream_t st);
hipError_t launch_pack_stream(const void* W, int N, int K, int ldw, void* Wp, hipStream_t st);
hipError_t launch_pack_kblock(const void* W, int N, int K, int ldw, void* Wb, hipStream_t st);

// 8-bit floating point variant (gemm_fp8.hip): E4M3 codes with one fp32 scale per row.
hipError_t launch_quantize_rows_f8(const void* x, int rows, int K, int ldx, void* q, int ldq,
                                   float* scale, hipStream_t st);
hipError_t launch_gemm_f8(const void* A, const float* sa, const void* W, const float* sw, void* C,
                          const void* R, int M, int N, int K, int lda, int ldw, int ldc, int epilogue,
                          hipStream_t st, const EpiArgs* ea = nullptr);

hipError_t launch_rope_table(float2* table, int n_pos, int head_dim, float theta, hipStream_t st);

// Batched pieces take per-sequence row offsets cu[batch+1] (device) of the current stage;
// cu == nullptr means one sequence of n_single rows (cu_vt likewise means offset 0).
hipError_t launch_embed(const void* embed, const int32_t* ids, const float* scale, const int32_t* cu,
                        int batch, int total, int d, int vocab, void* h, int32_t* pos,
                        int32_t* status, hipStream_t st, unsigned long long* ssq = nullptr);
hipError_t launch_rmsnorm(const void* h, const void* gain, void* x, int rows, int d, float eps,
                          hipStream_t st);
hipError_t launch_v_transpose(const void* v, void* vt, const int32_t* cu, const int32_t* cu_vt,
                              int n_single, int batch, int max_rows, int vt_ld, int n_heads,
                              int head_dim, hipStream_t st);
// Once per pruning stage: zeroes the columns of vt between each sequence's end and the next
// multiple of 64 (the attention kernel multiplies them by probabilities that are exactly 0,
// so they must be finite) and, for a packed batch, writes the column of every row.
hipError_t launch_vt_stage_setup(void* vt, int32_t* vt_col, const int32_t* cu, const int32_t* cu_vt,
                                 int n_single, int batch, int vt_ld, int n_feat, hipStream_t st);
hipError_t launch_attention(const void* q, const void* k, const void* vt, void* o, const int32_t* cu,
                            const int32_t* cu_vt, int n_single, int batch, int max_rows, int vt_ld,
                            int n_heads, int head_dim, hipStream_t st, float* z = nullptr,
                            void* zstat = nullptr, int z_ld = 0, int kv_group = 1);
// Eq. 1 from the logits the attention kernel left in `scratch` (z, zstat of launch_attention
// = score_z(scratch), score_zstat(scratch, z_ld, H); z_ld = vt_ld, sequence b at cu_vt[b]).
float* score_z(void* scratch);
void* score_zstat(void* scratch, int z_ld, int n_heads);
hipError_t launch_score_finish(float* s, void* scratch, const int32_t* cu, const int32_t* cu_z,
                               int n_single, int batch, int z_ld, int max_rows, int n_heads,
                               hipStream_t st);
size_t score_scratch_bytes(int total_rows, int batch, int n_heads);
hipError_t launch_score(const void* q, const void* k, float* s, void* scratch, const int32_t* cu,
                        int n_single, int batch, int total_rows, int max_rows, int n_heads,
                        int head_dim, hipStream_t st);
hipError_t launch_select(const float* s, const int32_t* cu_prev, const int32_t* cu_new,
                         int m_single, int k_single, int batch, int32_t* keep_idx,
                         int32_t* prune_idx, hipStream_t st);
hipError_t launch_gather(const void* h, const int32_t* pos, const int32_t* keep_idx, int n_keep,
                         const int32_t* prune_idx, int n_prune, void* h_out, int32_t* pos_out,
                         void* aux_h, int32_t* aux_pos, int d, hipStream_t st,
                         unsigned long long* ssq = nullptr);
hipError_t launch_final_norm(const void* h, const int32_t* cu, int n_single, int batch,
                             const void* gain, float* xf, int d, float eps, hipStream_t st);
hipError_t launch_lm_head(const float* xf, const void* w_lm, float* logits, int batch, int d,
                          int vocab, hipStream_t st);
bool lm_head_fused_fits(int batch, int d);
hipError_t launch_lm_head_fused(const void* h, const int32_t* cu, int n_single, int batch, const void* gain,
                                const void* w_lm, float* logits, int d, int vocab, float eps, hipStream_t st);

// ---- decoding steps (position-indexed generation state; see decode.hip) -----------------
// Bits of the device status word (the public header's LAZYLLM_ST_* values).
constexpr int ST_BAD_TOKEN = 1, ST_BAD_CU = 2, ST_NO_STATE = 4, ST_EXCHANGE = 8;
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st);
hipError_t launch_scatter_rows(const void* src, const int32_t* pos, int n, void* dst, uint8_t* flag,
                               int d, hipStream_t st);
hipError_t launch_scatter_vt(const void* v, const int32_t* pos, int n, int d, void* vt, int vt_ld,
                             hipStream_t st);
hipError_t launch_gen_embed(const void* embed, const int32_t* token_id, int vocab, int d, int new_pos,
                            void* h, unsigned long long* ssq, int32_t* run_pos, int32_t* live_row,
                            uint8_t* has_kv0, int32_t* status, hipStream_t st);
hipError_t launch_gen_stage(const float* s, const uint8_t* member_prev, int n_tot, int k,
                            uint8_t* member, unsigned long long* member_bits, uint8_t* has_kv,
                            uint8_t* has_aux, int32_t* live_row, int32_t* run_pos,
                            int32_t* src_row, int32_t* park_src, int32_t* park_pos,
                            int32_t* counts, int32_t* status, hipStream_t st);
hipError_t launch_revive_gather(const void* h_prev, void* aux, const int32_t* run_pos,
                                const int32_t* src_row, int n_rows, const int32_t* park_src,
                                const int32_t* park_pos, int n_park, void* h_new,
                                unsigned long long* ssq, int d, hipStream_t st);
hipError_t launch_decode_attention(const void* q, const int32_t* qpos, int M, const void* k,
                                   const void* vt, int vt_ld, const unsigned long long* sel_bits,
                                   int n_keys, void* o, int n_heads, int head_dim, hipStream_t st,
                                   float* z = nullptr, void* zstat = nullptr, int z_ld = 0,
                                   void* split_ws = nullptr, size_t split_ws_bytes = 0,
                                   int kv_group = 1);
size_t decode_attention_workspace_bytes(int d_model, int n_heads);
// the ticket counters at the end of that workspace must be zero before the first attention launch
hipError_t launch_decode_attention_counters_clear(void* split_ws, size_t split_ws_bytes, hipStream_t st);

struct PlanArgs {
  int32_t n_stages;                     // pruning stages after stage 0
  int32_t permille[128];                // keep ratio entering stage s+1
};
// cu_stage[(n_stages+1)][batch+1], cu_aux[n_stages][batch+1], cu_vt[(n_stages+1)][batch+1]
// seqlens_host[batch]: the lengths every buffer was sized from; they reach the device by value,
// LENS_PER_LAUNCH per launch.  cu_dev (may be null when batch == 1) is only checked against them.
constexpr int LENS_PER_LAUNCH = 960;
struct LensChunk {
  int32_t n[LENS_PER_LAUNCH];
};
hipError_t launch_plan(const int32_t* cu_dev, const int32_t* seqlens_host, int batch, int expect_total,
                       const PlanArgs& plan, int32_t* cu_stage, int32_t* cu_aux, int32_t* cu_vt,
                       int32_t* status, hipStream_t st);

// Weight repacking (model creation, off the hot path).
hipError_t launch_copy_rows(const void* src, void* dst, int rows, int cols, int src_ld, int dst_ld,
                            hipStream_t st);
hipError_t launch_scale_cols(void* w, const void* gain, size_t rows, int cols, hipStream_t st);
hipError_t launch_interleave_gate_up(const void* gate, const void* up, void* dst, int f, int f_pad,
                                     int d, hipStream_t st);

}  // namespace lz
