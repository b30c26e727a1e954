/*
 * lazyllm.h -- C ABI of the MI355X (gfx950) pruned-prefill library.
 *
 * Implements the prefilling stage of LazyLLM (arxiv 2407.14057, Sec. 3.1-3.2):
 * every decoder layer runs on the surviving prompt tokens only, each token is
 * scored by the head-averaged attention probability of the last token
 * attending to it (Eq. 1), pruning layers keep the top-k percentile of the
 * surviving tokens (Sec. 3.2, "Progressive Token Pruning"), hidden states and
 * position ids are compacted, and the hidden states of dropped tokens are
 * parked in an Aux Cache (Sec. 3.2, "Aux Cache").  Decoding steps after such a
 * prefill (lazyllm_decode_step) select afresh in every step and revive pruned
 * tokens from the Aux Cache.
 *
 * Conventions
 *   - "device" pointers are HIP device memory owned by the caller unless said
 *     otherwise; "host" pointers are ordinary process memory.
 *   - bf16 tensors are raw 16-bit patterns; matrices are row-major
 *     [out_features, in_features] (y = x W^T).
 *   - every call that enqueues work takes a hipStream_t as void*; work is
 *     asynchronous on that stream and the results are valid once the caller
 *     has synchronised it.  Nothing here synchronises except model_create
 *     and lazyllm_decode_step (once per pruning layer, see there).
 *   - return value 0 is success, negative values are lazyllm_status codes.
 *     No call throws or aborts.  Argument validation happens before the first
 *     HIP call, so the error paths can be exercised without a GPU.
 *   - one GPU, one stream per call.  Calls sharing a workspace or an output
 *     buffer must be ordered by the caller.
 */
#ifndef LAZYLLM_H
#define LAZYLLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LAZYLLM_MAX_LAYERS 128

typedef enum lazyllm_status {
  LAZYLLM_OK = 0,
  LAZYLLM_EINVAL = -1, /* bad argument (null pointer, size, schedule, shape) */
  LAZYLLM_ENOSPC = -2, /* workspace or output buffer too small */
  LAZYLLM_EHIP = -3,   /* HIP runtime failure; see lazyllm_last_hip_error() */
  LAZYLLM_ENOMEM = -4, /* host or device allocation failed in model_create */
  LAZYLLM_EFAILED = -5 /* the generation handle is unusable: an earlier step failed part-way */
} lazyllm_status;

/* Decoder shape (Sec. 3.1: a stack of layers, each multi-head self-attention
 * followed by an MLP; Llama 2 conventions: pre-norm RMSNorm, rotary position
 * embedding with half-split pairing, SwiGLU MLP, untied LM head, no biases).
 * Supported: head_dim 64 or 128, d_model == n_heads * head_dim,
 * d_model % 128 == 0, 1 <= n_layers <= LAZYLLM_MAX_LAYERS.
 * n_kv_heads: grouped-query attention as a model variant -- that many K,V
 * heads, each read by n_heads / n_kv_heads consecutive query heads; 0 means
 * n_heads (plain multi-head attention, the paper's models).  It must divide
 * n_heads and n_kv_heads * head_dim must be a multiple of 128.  Eq. 1 is the
 * mean over all n_heads attention maps either way.
 * gemm_dtype: arithmetic of the four projections of every layer in the
 * prefill.  0 = 16-bit floating point (bf16 storage, fp32 accumulation; the
 * paper's Sec. 4 names its hardware and framework but no precision, the
 * benchmark this library is measured on is quoted at bf16).  1 = the 8-bit variant (see lazyllm_op_gemm_fp8): the stored
 * weights (RMSNorm gains folded in) are quantised once at model creation,
 * the activations row by row in front of each projection, OFP8 E4M3 codes
 * with one fp32 scale per row; attention, normalisation, scoring, selection
 * and the LM head are unchanged.  It needs d_model % 256 == 0,
 * (d_model + 2 * n_kv_heads * head_dim) % 256 == 0 and d_ffn <= 16384.  The
 * decoding steps always compute in 16-bit floating point (one token row is
 * bound by streaming the weights, not by the matrix cores); on such a model
 * they continue from the K,V and Aux Cache the 8-bit prefill left. */
typedef struct lazyllm_config {
  int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
  float rms_eps, rope_theta;
  int32_t n_kv_heads;
  int32_t gemm_dtype;
} lazyllm_config;

/* Device pointers to bf16 weights.  The per-layer members are HOST arrays of
 * n_layers device pointers. */
typedef struct lazyllm_weights {
  const void* embed;              /* [vocab, d_model] */
  const void* const* attn_norm;   /* [d_model] each */
  const void* const* wq;          /* [d_model, d_model] */
  const void* const* wk;          /* [n_kv_heads * head_dim, d_model] */
  const void* const* wv;          /* [n_kv_heads * head_dim, d_model] */
  const void* const* wo;
  const void* const* ffn_norm;    /* [d_model] */
  const void* const* w_gate;      /* [d_ffn, d_model] */
  const void* const* w_up;        /* [d_ffn, d_model] */
  const void* const* w_down;      /* [d_model, d_ffn] */
  const void* final_norm;         /* [d_model] */
  const void* lm_head;            /* [vocab, d_model] */
} lazyllm_weights;

/* One pruning layer (Sec. 5.2's three knobs: how many pruning layers, where,
 * how much).  The scores of layer `layer`-1 decide which tokens enter
 * `layer`; keep_permille/1000 is the fraction kept of the tokens that ran
 * `layer`-1, counted as max(1, ceil(m * keep_permille / 1000)) in integer
 * arithmetic; the last token is always kept and is part of that count.
 * Entries must be sorted by strictly increasing layer, 1 <= layer < n_layers,
 * 0 < keep_permille <= 1000 (1000 = no pruning at that layer). */
typedef struct lazyllm_keep {
  int32_t layer;
  int32_t keep_permille;
} lazyllm_keep;

typedef struct lazyllm_model lazyllm_model;

/* Flags for lazyllm_prefill*. */
#define LAZYLLM_SCORE_ALL_LAYERS 0u   /* default: Eq. 1 scores for every layer */
#define LAZYLLM_SCORE_ONLY_USED 1u    /* only for layers whose successor prunes;
                                         result.scores of other layers is NULL */
#define LAZYLLM_KEEP_HIDDEN 2u        /* also return every layer's input hidden states and the
                                         last layer's output (verification aid; adds copies) */
#define LAZYLLM_FUSE_COMPACTION 4u    /* Sec. 3.2's gather folded into the next layer: the kept rows
                                         are not copied; the layer after a selection reads them
                                         through the index of kept rows (A operand and row scales
                                         of its QKV projection, residual of its O projection).
                                         Same bits as without.  Ignored with LAZYLLM_KEEP_HIDDEN
                                         and with gemm_dtype 1. */

/* Bits of *lazyllm_result.status (device int32, read after stream sync). */
#define LAZYLLM_ST_BAD_TOKEN 1       /* a token id was outside [0, vocab); clamped */
#define LAZYLLM_ST_BAD_CU 2          /* device cu_seqlens disagrees with the host copy */
#define LAZYLLM_ST_NO_STATE 4        /* decoding: a selected token had neither K,V nor an Aux Cache
                                        entry at a layer (the state buffer was damaged) */
#define LAZYLLM_ST_EXCHANGE 8        /* a matrix product whose workgroups hand partial sums to each
                                        other gave up on a hand-over (a workgroup was not resident,
                                        or not on the XCD it was expected on): the outputs of this
                                        call are not to be used */

/* Where the results of one prefill live.  Every pointer is device memory
 * inside the caller's output buffer and stays valid as long as that buffer.
 * Rows of all sequences are packed back to back; within a sequence rows are in
 * ascending original position.  Layers between two pruning layers share one
 * kept set, so their kept_pos / cu_kept pointers alias the same memory. */
typedef struct lazyllm_result {
  int32_t batch, n_layers;
  int32_t n_tokens[LAZYLLM_MAX_LAYERS]; /* rows that ran layer l, over the batch */
  float* logits;                        /* fp32 [batch, vocab], last token of each prompt */
  int32_t* kept_pos[LAZYLLM_MAX_LAYERS];/* int32 [n_tokens[l]] original position in its prompt */
  int32_t* cu_kept[LAZYLLM_MAX_LAYERS]; /* int32 [batch+1] row offsets per sequence */
  void* k[LAZYLLM_MAX_LAYERS];          /* bf16 [n_tokens[l], n_kv_heads, head_dim], rotary applied */
  void* v[LAZYLLM_MAX_LAYERS];          /* bf16 [n_tokens[l], n_kv_heads, head_dim] */
  float* scores[LAZYLLM_MAX_LAYERS];    /* fp32 [n_tokens[l]]  Eq. 1, or NULL */
  /* Aux Cache: only for layers that prune (NULL / 0 elsewhere).  Row i is a
   * token dropped on entry to layer l: its layer-l input hidden state and its
   * original position. */
  int32_t n_aux[LAZYLLM_MAX_LAYERS];
  void* aux_h[LAZYLLM_MAX_LAYERS];      /* bf16 [n_aux[l], d_model] */
  int32_t* aux_pos[LAZYLLM_MAX_LAYERS]; /* int32 [n_aux[l]] */
  int32_t* cu_aux[LAZYLLM_MAX_LAYERS];  /* int32 [batch+1] */
  int32_t* status;                      /* int32 [1] LAZYLLM_ST_* bits */
  /* Only with LAZYLLM_KEEP_HIDDEN (NULL otherwise): the residual stream entering layer l
   * (after that layer's compaction), bf16 [n_tokens[l], d_model], and the stream leaving the
   * last layer, bf16 [n_tokens[n_layers-1], d_model]. */
  void* hidden_in[LAZYLLM_MAX_LAYERS];
  void* hidden_out;
} lazyllm_result;

/* ---- host-only helpers (no HIP call) ------------------------------------------------ */

/* Tokens that run each layer for a prompt of n tokens under the schedule
 * (Sec. 3.2: kept sets are nested, so the counts never grow).
 * n_per_layer: host int32[n_layers].  EINVAL on a bad schedule or n <= 0. */
int lazyllm_keep_counts(int32_t n, int32_t n_layers, const lazyllm_keep* sched, int32_t n_sched,
                        int32_t* n_per_layer);

/* Bytes of scratch a prefill of `total_tokens` rows in `batch` sequences, the
 * longest `max_seqlen` tokens, needs.  0 on a bad argument. */
size_t lazyllm_workspace_bytes(const lazyllm_config* cfg, int32_t total_tokens, int32_t batch,
                               int32_t max_seqlen);

/* Bytes of output buffer for these prompt lengths (host int32[batch]), schedule
 * and prefill flags.  0 on a bad argument. */
size_t lazyllm_output_bytes(const lazyllm_config* cfg, const int32_t* seqlens, int32_t batch,
                            const lazyllm_keep* sched, int32_t n_sched, uint32_t flags);

const char* lazyllm_strerror(int status);
/* hipError_t value of the last failing HIP call on this thread (0 if none). */
int lazyllm_last_hip_error(void);
/* Library ABI version, bumped on any signature change. */
int lazyllm_abi_version(void);

/* ---- model ---------------------------------------------------------------------------- */

/* Copies the weights into the library's own MFMA-friendly layout (fused QKV,
 * gate/up interleaved in 32-row blocks, d_ffn zero-padded to a multiple of
 * 128; the RMSNorm gains multiplied into the columns of the QKV and gate/up
 * matrices, which is exact for gains of 1 and one more bf16 rounding of the
 * weight otherwise).  Allocates device memory (about the size of the weights), runs the
 * repack on `hip_stream` and synchronises it: after return the caller's
 * weight buffers are no longer referenced.  *out is set only on success. */
int lazyllm_model_create(const lazyllm_config* cfg, const lazyllm_weights* w, void* hip_stream,
                         lazyllm_model** out);
void lazyllm_model_destroy(lazyllm_model* m);

/* ---- the prefill (Sec. 3.1 prefilling stage with Sec. 3.2 pruning) -------------------- */

/* One prompt of n tokens.  token_ids: device int32[n].  embed_scale: device
 * fp32[n] multiplying each token's embedding row, or NULL.  workspace /
 * out_buf: device, 256-byte aligned, at least lazyllm_workspace_bytes /
 * lazyllm_output_bytes.  res: host struct filled before return (its pointers
 * point into out_buf).  Enqueues everything on hip_stream and returns. */
int lazyllm_prefill(const lazyllm_model* m, const int32_t* token_ids, const float* embed_scale,
                    int32_t n, const lazyllm_keep* sched, int32_t n_sched, uint32_t flags,
                    void* workspace, size_t ws_bytes, void* out_buf, size_t out_bytes,
                    void* hip_stream, lazyllm_result* res);

/* `batch` independent prompts packed back to back; each is pruned on its own
 * with the same schedule.  cu_seqlens_host: host int32[batch+1], starting at 0,
 * strictly increasing.  cu_seqlens_dev: the same values in device memory (may be NULL when
 * batch == 1).  Every buffer, launch and row table follows the host copy; the device copy is only
 * compared with it on the GPU, and a difference sets LAZYLLM_ST_BAD_CU in *status (the result is
 * then the one the host copy describes). */
int lazyllm_prefill_varlen(const lazyllm_model* m, const int32_t* token_ids,
                           const float* embed_scale, const int32_t* cu_seqlens_host,
                           const int32_t* cu_seqlens_dev, int32_t batch, const lazyllm_keep* sched,
                           int32_t n_sched, uint32_t flags, void* workspace, size_t ws_bytes,
                           void* out_buf, size_t out_bytes, void* hip_stream, lazyllm_result* res);

/* ---- decoding steps with the Aux Cache (Sec. 3.2, "Aux Cache") ---------------------------
 *
 * After a pruned prefill the KV cache of layer l holds only the tokens that ran layer l.
 * Every decoding step selects afresh: the new token's attention row gives Eq. 1's scores,
 * each pruning layer keeps the top-k percentile of the tokens selected at the layer below
 * (same rule and schedule as the prefill, counted over all tokens so far; the new token is
 * forced), and a token pruned earlier may be selected again.  A selected token whose K,V
 * exist at the layer is read from the cache.  One whose K,V are missing is revived: its
 * layer input is the hidden state it carries out of the layer below in this step, or else the
 * Aux Cache entry of this layer; it runs the layer like the new token (its attention sees the
 * selected tokens at or before its own position) and its K,V stay in the cache, so no token
 * is computed twice in a layer.  A token that carries a state but is not selected at a
 * pruning layer leaves that state in the layer's Aux Cache.
 *
 * The generation state lives in ONE caller-owned device buffer and is indexed by original
 * position (capacity = prompt length + the most tokens that will be generated):
 *   per layer   K  bf16 [capacity, kv_dim]             row p = token at position p
 *               Vt bf16 [kv_dim, vt_ld]                column p (V transposed, vt_ld = capacity
 *                                                      rounded up to 64; kv_dim = n_kv_heads *
 *                                                      head_dim, = d_model without shared heads)
 *   per pruning layer and the layers up to the next one (they share one set of tokens)
 *               has_kv  uint8 [capacity]               1 where K,V exist
 *   per pruning layer
 *               aux_h   bf16 [capacity, d_model], has_aux uint8 [capacity]
 * Rows never written are zero.  The schedule is fixed when the state is made. */
typedef struct lazyllm_generation lazyllm_generation;

typedef struct lazyllm_generation_view {
  int32_t n_layers, capacity, n_prompt, n_tokens, vt_ld;
  void* k[LAZYLLM_MAX_LAYERS];
  void* vt[LAZYLLM_MAX_LAYERS];
  uint8_t* has_kv[LAZYLLM_MAX_LAYERS];   /* layers of one stage alias the same table */
  void* aux_h[LAZYLLM_MAX_LAYERS];       /* pruning layers only, NULL elsewhere */
  uint8_t* has_aux[LAZYLLM_MAX_LAYERS];
} lazyllm_generation_view;

/* What one step did.  logits and status live in the state buffer; the per-layer
 * tables live in the step's workspace and are overwritten by the next step. */
typedef struct lazyllm_step_result {
  int32_t n_layers;
  int32_t n_tokens;                           /* tokens so far, this step's included */
  int32_t position;                           /* original position of this step's token */
  float* logits;                              /* fp32 [vocab]: distribution of the NEXT token */
  int32_t n_selected[LAZYLLM_MAX_LAYERS];     /* tokens attended at layer l in this step */
  int32_t n_ran[LAZYLLM_MAX_LAYERS];          /* tokens that ran layer l (new token + revived) */
  const uint8_t* selected[LAZYLLM_MAX_LAYERS];/* uint8 [n_tokens] membership by position; NULL = all */
  const int32_t* ran_pos[LAZYLLM_MAX_LAYERS]; /* int32 [n_ran[l]] ascending; last = new token */
  float* scores[LAZYLLM_MAX_LAYERS];          /* fp32 [n_tokens] Eq. 1 by position, 0 if not selected */
  int32_t* status;                            /* int32 [1] LAZYLLM_ST_* bits (accumulates) */
} lazyllm_step_result;

/* Bytes of the state buffer / of one step's workspace.  0 on a bad argument. */
size_t lazyllm_generation_state_bytes(const lazyllm_config* cfg, const lazyllm_keep* sched,
                                      int32_t n_sched, int32_t capacity);
size_t lazyllm_decode_workspace_bytes(const lazyllm_config* cfg, const lazyllm_keep* sched,
                                      int32_t n_sched, int32_t capacity);

/* Builds the state from the result of a single-prompt lazyllm_prefill made with the same
 * schedule: zeroes `state` (device, 256-byte aligned, >= lazyllm_generation_state_bytes),
 * scatters the packed K, V and Aux Cache rows to their positions.  Enqueued on hip_stream, not
 * synchronised; the prefill's output buffer may be released once the stream has passed this
 * work.  Allocates a few bytes of pinned host memory for the handle.  capacity must exceed
 * the prompt length.  EINVAL if the result does not match model and schedule. */
int lazyllm_generation_create(const lazyllm_model* m, const lazyllm_keep* sched, int32_t n_sched,
                              int32_t capacity, const lazyllm_result* prefill, void* state,
                              size_t state_bytes, void* hip_stream, lazyllm_generation** out);
void lazyllm_generation_destroy(lazyllm_generation* g);
/* Pointers into the state buffer (host call, no HIP). */
int lazyllm_generation_get_view(const lazyllm_generation* g, lazyllm_generation_view* v);

/* One decoding step on the token *token_id (device int32[1]), which takes the next
 * position.  Returns res->logits for the token after it.  workspace: device, 256-byte
 * aligned, >= lazyllm_decode_workspace_bytes.  Unlike the prefill this call SYNCHRONISES
 * hip_stream once per pruning layer: the number of revived tokens is data-dependent and sets
 * the shape of every launch that follows.  The layers after the last pruning layer are
 * still in flight at return.  ENOSPC when the capacity is used up (the state is untouched and
 * stays usable, as after EINVAL).  A step that fails after its first launch (EHIP) has already
 * changed the state without advancing the token count: the handle is marked failed, every
 * later step returns LAZYLLM_EFAILED, and the only valid call left is
 * lazyllm_generation_destroy. */
int lazyllm_decode_step(lazyllm_generation* g, const int32_t* token_id, void* workspace,
                        size_t ws_bytes, void* hip_stream, lazyllm_step_result* res);

/* ---- per-launch timing of the prefill (measurement aid) --------------------------------
 * Between profile_begin and profile_end every kernel launch of lazyllm_prefill* is
 * bracketed by hipEvents on the call's stream.  profile_end waits for the recorded work,
 * then writes up to `capacity` records (launch order) and the total count.  `work` is the
 * launch's algorithmic work: FLOPs for the GEMM and attention steps (Sec. 5.3: linear layers
 * grow linearly, attention quadratically with the tokens computed), bytes for the
 * bandwidth-bound steps.  Not thread-safe; one stream at a time.
 * Steps without a launch of their own never appear: RMSNorm is folded into the QKV and gate/up
 * GEMMs, Eq. 1's finish rides in the gate/up launch, and V_TRANSPOSE is only the once-per-stage
 * zeroing of the transposed V buffer's padding (the copy itself is part of the QKV epilogue). */
enum lazyllm_step {
  LAZYLLM_STEP_PLAN = 0, LAZYLLM_STEP_ROPE_TABLE, LAZYLLM_STEP_EMBED, LAZYLLM_STEP_SELECT,
  LAZYLLM_STEP_GATHER, LAZYLLM_STEP_RMSNORM, LAZYLLM_STEP_GEMM_QKV, LAZYLLM_STEP_V_TRANSPOSE,
  LAZYLLM_STEP_SCORE, LAZYLLM_STEP_ATTENTION, LAZYLLM_STEP_GEMM_O, LAZYLLM_STEP_GEMM_GATE_UP,
  LAZYLLM_STEP_GEMM_DOWN, LAZYLLM_STEP_LM_HEAD, LAZYLLM_STEP_COUNT
};
typedef struct lazyllm_profile_record {
  int32_t step;   /* lazyllm_step */
  int32_t layer;  /* -1 outside the layer loop */
  int32_t rows;   /* token rows the launch worked on */
  float ms;       /* event-to-event time */
  double work;    /* FLOPs or bytes, see above */
} lazyllm_profile_record;
int lazyllm_profile_begin(void);
int lazyllm_profile_end(lazyllm_profile_record* out, int32_t capacity, int32_t* n_records);

/* ---- single steps of the path (used by kernel-level parity tests and roofline
 *      measurements; all pointers device, all work enqueued on hip_stream) -------------- */

/* C[M,N] = A[M,K] W[N,K]^T in bf16 with fp32 accumulation (the linear layers
 * of Sec. 3.1's attention and MLP blocks).  lda/ldw/ldc are row strides in
 * elements.  epilogue 0: C = bf16(acc).  epilogue 1: C = bf16(R + acc) with
 * R[M,N] (row stride ldc) the residual stream; C may alias R.
 * epilogue 2 (SwiGLU): W holds gate and up rows interleaved in blocks of 32
 * (rows 64j..64j+31 gate, 64j+32..64j+63 up), C[M,N/2] = silu(gate) * up.
 * Requires N % 128 == 0, K % 64 == 0, 16-byte aligned rows.
 * workspace: optional device scratch of lazyllm_op_gemm_workspace_bytes() (256-byte
 * aligned) that lets epilogues 0 and 1 use the stream-K schedule for shapes whose tile
 * count does not divide over the CUs, and epilogue 2 walk its tiles with one workgroup per
 * CU when there are more tiles than CUs (same bits either way); NULL = never.
 * Bits 8..15 of `epilogue` force a tile configuration (measurement hook; 0 = the
 * library chooses): 2 = 128x128, 3 = 128x128 in waves of 32x128, 4 = 128x256, 5 = 256x256 ping-pong, 7 = 192x256
 * ping-pong, 6 = 128x128 stream-K (needs the workspace), 8 = the weight-streaming
 * kernel of the decoding steps (M <= 32, needs the workspace), 9 / 10 = the 256x256 / 192x256
 * ping-pong tiles under the persistent stream-K schedule (need the workspace), 13 = 128x256 on
 * 8 waves of 32x128 with three stages, 14 = 256x256 on four waves of 128x128 (one per SIMD).  EINVAL where a
 * configuration does not fit the shape. */
size_t lazyllm_op_gemm_workspace_bytes(void);
int lazyllm_op_gemm(const void* A, const void* W, void* C, const void* R, int32_t M, int32_t N,
                    int32_t K, int32_t lda, int32_t ldw, int32_t ldc, int32_t epilogue,
                    void* workspace, size_t ws_bytes, void* hip_stream);

/* lazyllm_op_gemm with RMSNorm (the pre-norm of Sec. 3.1's Llama blocks) folded in, the form
 * the prefill runs.  ssq: uint64 [M], a row's sum of squares in 2^-32 fixed point.
 *  - ssq_in (epilogues 0 and 2): row t of the product is multiplied by
 *    rsqrt(ssq_in[t] * 2^-32 / K + eps), i.e. C = rmsnorm(A) W^T for a gain of 1 (a gain is
 *    folded into W's columns by the caller).
 *  - ssq_out (epilogue 1): the sum of squares of each row of C as written (bf16) is ADDED to
 *    ssq_out[t] by integer atomics (order-independent); the caller zeroes it beforehand, or
 *    passes the same buffer as another call's ssq_clear.
 *  - ssq_clear: rows 0..M-1 of this buffer are set to zero.
 * Any of the three may be NULL.  workspace as for lazyllm_op_gemm; with ssq_in or ssq_clear it
 * is used by epilogue 2 only (the schedules open to the other two do not scale or clear rows). */
int lazyllm_op_gemm_rmsnorm(const void* A, const void* W, void* C, const void* R, int32_t M,
                            int32_t N, int32_t K, int32_t lda, int32_t ldw, int32_t ldc,
                            int32_t epilogue, const uint64_t* ssq_in, float eps, uint64_t* ssq_out,
                            uint64_t* ssq_clear, void* workspace, size_t ws_bytes,
                            void* hip_stream);

/* Weight layout of the tile kernels inside the model (for measurement and tests).  W [N, K] bf16
 * (device, row stride ldw elements) is rewritten K-step-major into `packed` (N * K * 2 bytes,
 * device, 16-byte aligned): [K / 64][N][64], i.e. the 128 bytes of one 64-element K step of all
 * rows one after the other, so that the W slab a tile needs for one step is one contiguous run
 * instead of one cache line from each of 256 rows.  K % 64 == 0.  lazyllm_op_gemm reads such a
 * weight when bit 29 of `epilogue` is set (ldw is then ignored; every tile configuration, not
 * configuration 8). */
int lazyllm_op_pack_weight_ksteps(const void* W, int32_t N, int32_t K, int32_t ldw, void* packed,
                                  void* hip_stream);

/* Weight layout of the decoding steps' weight-streaming kernel (for callers that cannot change
 * the model: measurement and tests).  W [N, K] bf16 (device, row stride ldw elements) is rewritten
 * into `packed` (N * K * 2 bytes, device, 16-byte aligned): for every group of 128 output
 * features and every 32-element K step the 8 KB that the kernel copies into one LDS slot, stored
 * contiguously, steps of a group one after the other -- each wave then reads one sequential
 * stream.  N % 128 == 0, K % 64 == 0.  lazyllm_op_gemm reads such a weight when bit 30 of
 * `epilogue` is set together with the forced configuration 8 (ldw is then ignored). */
int lazyllm_op_pack_weight_stream(const void* W, int32_t N, int32_t K, int32_t ldw, void* packed,
                                  void* hip_stream);

/* ---- 8-bit floating point variant of the projections' GEMM --------------------------------
 * An extension for the gfx950 8-bit matrix instructions; it is not the paper's arithmetic (its
 * Sec. 4 names hardware and framework only) and never the arithmetic of the headline figure.
 * Operands are OFP8 E4M3 codes (OCP 8-bit Floating Point Specification: bias 7, no infinities,
 * S.1111.111 = NaN, largest value 448) with one fp32 scale per row, both K-contiguous.
 *
 * lazyllm_op_quantize_fp8: x [rows, K] bf16 (device, row stride ldx elements, 16-byte aligned)
 *   -> codes [rows, K] uint8 (device, row stride ldq bytes, 8-byte aligned) and scale [rows] fp32
 *   (device): scale = max|row| / 448 in fp32 (1 for an all-zero row), code = E4M3(x / scale) with
 *   the division in fp32, round to nearest, ties to even, saturating.  K % 8 == 0, K <= 16384,
 *   ldx % 8 == 0, ldq % 8 == 0; inputs must be finite.  One pass over x.
 *
 * lazyllm_op_gemm_fp8: C[m, n] = a_scale[m] * w_scale[n] * sum_k a[m, k] * w[n, k], accumulated in
 *   fp32, then the epilogue (0 store, 1 + R, 2 SiLU(gate)*up over interleaved columns, as in
 *   lazyllm_op_gemm), written as bf16.  a_codes [M, K] and w_codes [N, K] are E4M3 codes (device,
 *   16-byte aligned, row strides lda, ldw bytes, multiples of 16); w_scale 16-byte aligned.
 *   N % 256 == 0, K % 128 == 0, M * lda and N * ldw below 2^32.  C, R as in lazyllm_op_gemm.
 *   Bit 29 of `epilogue`: w_codes is K-step-major, [K / 128][N][128] (the form the model keeps;
 *   lazyllm_op_pack_weight_ksteps on the codes taken as N rows of K / 2 16-bit units); ldw is
 *   then ignored.
 * Both return LAZYLLM_EINVAL for arguments outside these limits; nothing is allocated and
 * nothing is kept. */
int lazyllm_op_quantize_fp8(const void* x, int32_t rows, int32_t K, int32_t ldx, void* codes,
                            int32_t ldq, float* scale, void* hip_stream);
int lazyllm_op_gemm_fp8(const void* a_codes, const float* a_scale, const void* w_codes,
                        const float* w_scale, void* C, const void* R, int32_t M, int32_t N, int32_t K,
                        int32_t lda, int32_t ldw, int32_t ldc, int32_t epilogue, void* hip_stream);

/* x = h * rsqrt(mean(h^2) + eps) * gain, bf16 in and out, rows of width d. */
int lazyllm_op_rmsnorm(const void* h, const void* gain, void* x, int32_t rows, int32_t d,
                       float eps, void* hip_stream);

/* Fused QKV projection with rotary embedding: [q|k|v] = x Wqkv^T with Wqkv bf16
 * [3*H*hd, H*hd] (q rows, then k, then v); q and k are rotated at pos[rows]
 * (original positions; half-split pairing, angle pos * theta^(-2i/hd)) in fp32
 * and rounded to bf16 once.  x, q, k, v: bf16 [rows, H*hd].
 * rope_table: device float2 scratch [max_pos+1, hd/2], filled by this call. */
int lazyllm_op_qkv_rope(const void* x, const void* wqkv, const int32_t* pos, int32_t max_pos,
                        void* rope_table, void* q, void* k, void* v, int32_t rows, int32_t n_heads,
                        int32_t head_dim, float theta, void* hip_stream);

/* Transposed copy vt[H, hd, vt_ld] of v[rows, H, hd] that the attention kernel
 * reads (columns rows..roundup(rows,64)-1 are zeroed; vt_ld % 64 == 0). */
int lazyllm_op_v_transpose(const void* v, void* vt, int32_t vt_ld, int32_t rows, int32_t n_heads,
                           int32_t head_dim, void* hip_stream);

/* Causal multi-head attention over one sequence of `rows` tokens in compacted
 * order (ascending original position, so compacted-causal = original-causal):
 * o = softmax(q k^T / sqrt(hd) + causal) v.  q, k: bf16 [rows, H, hd];
 * vt: bf16 [H, hd, vt_ld]; o: bf16 [rows, H*hd]. */
int lazyllm_op_attention(const void* q, const void* k, const void* vt, int32_t vt_ld, void* o,
                         int32_t rows, int32_t n_heads, int32_t head_dim, void* hip_stream);

/* lazyllm_op_attention plus Eq. 1 in the form the prefill uses: the attention
 * kernel leaves the last query's logits against every key in `scratch`, and a
 * second kernel turns them into s[j] = (1/H) sum_h softmax_j(...) (fp32 [rows]).
 * scratch: device, at least lazyllm_op_score_scratch_bytes(rows, H). */
int lazyllm_op_attention_score(const void* q, const void* k, const void* vt, int32_t vt_ld, void* o,
                               float* s, void* scratch, int32_t rows, int32_t n_heads,
                               int32_t head_dim, void* hip_stream);

/* Eq. 1: s[j] = (1/H) sum_h softmax_j(q_last[h] . k[j,h] / sqrt(hd)) over the
 * `rows` tokens present.  q_last: bf16 [H, hd] (the last token's rotated
 * query); k: bf16 [rows, H, hd]; s: fp32 [rows].
 * scratch: device, at least lazyllm_op_score_scratch_bytes(rows, H). */
size_t lazyllm_op_score_scratch_bytes(int32_t rows, int32_t n_heads);
int lazyllm_op_score(const void* q_last, const void* k, float* s, void* scratch, int32_t rows,
                     int32_t n_heads, int32_t head_dim, void* hip_stream);

/* lazyllm_op_score for callers that cannot allocate device memory or pass a scratch buffer:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, kernels and results as lazyllm_op_score, but the scratch (per-head logits and
 * softmax statistics) lives in a device array that is part of the library image,
 * LAZYLLM_SCORE_STATIC_SCRATCH_BYTES per GPU, held until the process ends.  The call allocates
 * nothing, frees nothing and does not synchronise; the device of `hip_stream` must be current.
 * LAZYLLM_ENOSPC when lazyllm_op_score_scratch_bytes(rows, n_heads) exceeds the array (e.g.
 * 32 heads: up to about 39 000 rows; 64 heads: about 19 000); nothing is truncated.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 * streams or threads) race and must be ordered by the caller.  Nothing in the array needs to
 * start at zero, so a call is not affected by what an earlier, larger call left there. */
#define LAZYLLM_SCORE_STATIC_SCRATCH_BYTES (6u * 1024u * 1024u)
int lazyllm_op_score_static(const void* q_last, const void* k, float* s, int32_t rows,
                            int32_t n_heads, int32_t head_dim, void* hip_stream);

/* Top-k percentile rule (Sec. 3.2): of m tokens with scores s keep the last
 * one and the k-1 best others (higher fp32 score first, then lower index).
 * keep_idx: int32 [k] ascending; prune_idx: int32 [m-k] ascending. */
int lazyllm_op_select(const float* s, int32_t m, int32_t k, int32_t* keep_idx, int32_t* prune_idx,
                      void* hip_stream);

/* Compaction and Aux Cache write: h_out[i] = h[keep_idx[i]], pos_out likewise;
 * aux_h[i] = h[prune_idx[i]], aux_pos likewise.  Rows are bf16 of width d. */
int lazyllm_op_gather(const void* h, const int32_t* pos, const int32_t* keep_idx, int32_t n_keep,
                      const int32_t* prune_idx, int32_t n_prune, void* h_out, int32_t* pos_out,
                      void* aux_h, int32_t* aux_pos, int32_t d, void* hip_stream);

/* logits[V] = rmsnorm(h_last, gain) . W_lm^T, fp32 out; xf: device fp32[d] scratch (written only
 * by the two-launch form that rows wider than 32768 elements take). */
int lazyllm_op_lm_head(const void* h_last, const void* gain, const void* w_lm, float* xf,
                       float* logits, int32_t d, int32_t vocab, float eps, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* LAZYLLM_H */
