// Host side of the C ABI: argument validation (before any HIP call), buffer layout, the
// model's repacked weights, and the per-layer launch sequence of the pruned prefill.
#include <stdlib.h>
#include <string.h>

#include <new>
#include <algorithm>
#include <vector>

#include "../../include/lazyllm.h"
#include "common.h"

using namespace lz;

namespace {

thread_local int g_last_hip_error = 0;

inline int hip_fail(hipError_t e) {
  g_last_hip_error = (int)e;
  return LAZYLLM_EHIP;
}
#define LZ_HIP(expr)                           \
  do {                                         \
    hipError_t e_ = (expr);                    \
    if (e_ != hipSuccess) return hip_fail(e_); \
  } while (0)

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// ---- optional per-launch timing (hipEvents around every launch of a prefill) ---------------
struct ProfRec {
  hipEvent_t start, stop;
  int step, layer, rows;
  double work;        // algorithmic FLOPs (MFMA steps) or bytes (bandwidth steps)
};
struct ProfState {
  bool on = false;
  std::vector<ProfRec> recs;
  std::vector<hipEvent_t> pool;
};
ProfState g_prof;

hipEvent_t prof_event() {
  if (!g_prof.pool.empty()) {
    hipEvent_t e = g_prof.pool.back();
    g_prof.pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

// Runs `expr` (a launch returning hipError_t); with profiling on, brackets it with events.
#define LZ_RUN(step_, layer_, rows_, work_, expr)                                      \
  do {                                                                                 \
    if (g_prof.on) {                                                                   \
      ProfRec r_;                                                                      \
      r_.start = prof_event(); r_.stop = prof_event();                                 \
      r_.step = (step_); r_.layer = (layer_); r_.rows = (rows_); r_.work = (work_);    \
      if (r_.start == nullptr || r_.stop == nullptr) return hip_fail(hipErrorUnknown); \
      LZ_HIP(hipEventRecord(r_.start, st));                                            \
      LZ_HIP(expr);                                                                    \
      LZ_HIP(hipEventRecord(r_.stop, st));                                             \
      g_prof.recs.push_back(r_);                                                       \
    } else {                                                                           \
      LZ_HIP(expr);                                                                    \
    }                                                                                  \
  } while (0)

bool config_ok(const lazyllm_config* c) {
  if (c == nullptr) return false;
  if (c->n_layers < 1 || c->n_layers > LAZYLLM_MAX_LAYERS) return false;
  if (c->head_dim != 64 && c->head_dim != 128) return false;
  if (c->n_heads < 1 || c->n_heads > 256) return false;
  if ((int64_t)c->n_heads * c->head_dim != c->d_model) return false;
  if (c->d_model % 128 != 0 || c->d_model > 16384) return false;
  // grouped-query attention: n_kv_heads K,V heads, each shared by n_heads / n_kv_heads query
  // heads (0 = n_heads); the K,V width must be a multiple of 128 like d_model
  if (c->n_kv_heads < 0 || c->n_kv_heads > c->n_heads) return false;
  if (c->n_kv_heads > 0 && (c->n_heads % c->n_kv_heads != 0 || (c->n_kv_heads * c->head_dim) % 128 != 0))
    return false;
  if (c->d_ffn < 1 || c->vocab < 1) return false;
  if (!(c->rms_eps > 0.f) || !(c->rope_theta > 0.f)) return false;
  if (c->gemm_dtype != 0 && c->gemm_dtype != 1) return false;
  if (c->gemm_dtype == 1) {
    // the 8-bit tile kernel works on 256 x 256 tiles and 128-element K steps; the row quantiser
    // holds a row of up to 16384 elements
    const int kvd = (c->n_kv_heads > 0 ? c->n_kv_heads : c->n_heads) * c->head_dim;
    if (c->d_model % 256 != 0 || (c->d_model + 2 * kvd) % 256 != 0 || c->d_ffn > 16384) return false;
  }
  return true;
}

inline int ffn_padded(int f) { return (f + 127) / 128 * 128; }
inline int kv_heads(const lazyllm_config* c) { return c->n_kv_heads > 0 ? c->n_kv_heads : c->n_heads; }
inline int kv_dim(const lazyllm_config* c) { return kv_heads(c) * c->head_dim; }

bool schedule_ok(int n_layers, const lazyllm_keep* sched, int n_sched) {
  if (n_sched < 0 || n_sched > LAZYLLM_MAX_LAYERS) return false;
  if (n_sched > 0 && sched == nullptr) return false;
  int prev = 0;
  for (int i = 0; i < n_sched; ++i) {
    if (sched[i].layer < 1 || sched[i].layer >= n_layers) return false;   // layer 0 has no prior scores
    if (sched[i].layer <= prev) return false;                             // sorted, no duplicates
    if (sched[i].keep_permille <= 0 || sched[i].keep_permille > 1000) return false;
    prev = sched[i].layer;
  }
  return true;
}

inline int keep_count(int m, int permille) {
  long long k = ((long long)m * permille + 999) / 1000;
  return k < 1 ? 1 : (int)k;
}

// Stage table: stage 0 = the full prompt; every schedule entry with permille < 1000 opens a
// new stage at its layer.
struct Stages {
  int n_stages = 1;                       // including stage 0
  int first_layer[LAZYLLM_MAX_LAYERS + 1];
  int permille[LAZYLLM_MAX_LAYERS + 1];
  int stage_of_layer[LAZYLLM_MAX_LAYERS];
  long long total[LAZYLLM_MAX_LAYERS + 1];   // rows over the batch
  int max_rows[LAZYLLM_MAX_LAYERS + 1];      // longest sequence
  long long vt_ld[LAZYLLM_MAX_LAYERS + 1];   // sum of per-sequence lengths rounded up to 64
};

void build_stages(int n_layers, const lazyllm_keep* sched, int n_sched, const int32_t* seqlens,
                  int batch, Stages* st) {
  st->n_stages = 1;
  st->first_layer[0] = 0;
  st->permille[0] = 1000;
  for (int i = 0; i < n_sched; ++i) {
    if (sched[i].keep_permille >= 1000) continue;
    st->first_layer[st->n_stages] = sched[i].layer;
    st->permille[st->n_stages] = sched[i].keep_permille;
    st->n_stages++;
  }
  int s = 0;
  for (int l = 0; l < n_layers; ++l) {
    if (s + 1 < st->n_stages && st->first_layer[s + 1] == l) ++s;
    st->stage_of_layer[l] = s;
  }
  for (int k = 0; k < st->n_stages; ++k) { st->total[k] = 0; st->max_rows[k] = 0; st->vt_ld[k] = 0; }
  for (int b = 0; b < batch; ++b) {
    int n = seqlens[b];
    for (int k = 0; k < st->n_stages; ++k) {
      if (k > 0) n = keep_count(n, st->permille[k]);
      st->total[k] += n;
      st->vt_ld[k] += (n + 63) / 64 * 64;
      if (n > st->max_rows[k]) st->max_rows[k] = n;
    }
  }
}

// ---- workspace layout -------------------------------------------------------------------
struct Workspace {
  size_t h0, h1, ssq0, ssq1, q, o, vt, vt_col, act, score, rope, keep_idx, prune_idx, xf, gemm_ws, a8, sa8, total;
};

void layout_workspace(const lazyllm_config* c, long long T, int batch, int max_seqlen,
                      Workspace* w) {
  const size_t d = c->d_model, fp = ffn_padded(c->d_ffn);
  const size_t vt_ld = (size_t)T + 64 * (size_t)batch;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
  w->h0 = take((size_t)T * d * 2);
  w->h1 = take((size_t)T * d * 2);
  w->ssq0 = take((size_t)T * 8);          // per row sum of squares of h (2^-32 fixed point), two roles
  w->ssq1 = take((size_t)T * 8);
  w->q = take((size_t)T * d * 2);
  w->o = take((size_t)T * d * 2);
  w->vt = take((size_t)kv_dim(c) * vt_ld * 2);
  w->vt_col = take((size_t)T * 4);
  w->act = take((size_t)T * fp * 2);
  w->score = take(score_scratch_bytes((int)T, batch, c->n_heads));
  w->rope = take((size_t)max_seqlen * (c->head_dim / 2) * sizeof(float2));
  w->keep_idx = take((size_t)T * 4);
  w->prune_idx = take((size_t)T * 4);
  w->xf = take((size_t)batch * d * 4);
  w->gemm_ws = take(gemm_workspace_bytes());
  // 8-bit variant: the codes and row scales of the activations in front of a projection
  w->a8 = take(c->gemm_dtype == 1 ? (size_t)T * (d > fp ? d : fp) : 0);
  w->sa8 = take(c->gemm_dtype == 1 ? (size_t)T * 4 : 0);
  w->total = off;
}

// ---- output layout ------------------------------------------------------------------------
struct Output {
  size_t status, cu_stage, cu_aux, cu_vt, logits;
  size_t kept_pos[LAZYLLM_MAX_LAYERS + 1];            // per stage
  size_t aux_h[LAZYLLM_MAX_LAYERS + 1], aux_pos[LAZYLLM_MAX_LAYERS + 1];
  size_t k[LAZYLLM_MAX_LAYERS], v[LAZYLLM_MAX_LAYERS], scores[LAZYLLM_MAX_LAYERS];
  size_t hidden_in[LAZYLLM_MAX_LAYERS], hidden_out;
  size_t total;
};

void layout_output(const lazyllm_config* c, const Stages* st, int batch, uint32_t flags, Output* o) {
  const size_t d = c->d_model;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t r = off; off += align_up(bytes); return r; };
  o->status = take(4);
  o->cu_stage = take((size_t)st->n_stages * (batch + 1) * 4);
  o->cu_aux = take((size_t)st->n_stages * (batch + 1) * 4);
  o->cu_vt = take((size_t)st->n_stages * (batch + 1) * 4);
  o->logits = take((size_t)batch * c->vocab * 4);
  for (int s = 0; s < st->n_stages; ++s) {
    o->kept_pos[s] = take((size_t)st->total[s] * 4);
    if (s > 0) {
      const size_t na = (size_t)(st->total[s - 1] - st->total[s]);
      o->aux_h[s] = take(na * d * 2);
      o->aux_pos[s] = take(na * 4);
    }
  }
  for (int l = 0; l < c->n_layers; ++l) {
    const size_t n = (size_t)st->total[st->stage_of_layer[l]];
    o->k[l] = take(n * (size_t)kv_dim(c) * 2);
    o->v[l] = take(n * (size_t)kv_dim(c) * 2);
    o->scores[l] = take(n * 4);
  }
  if (flags & LAZYLLM_KEEP_HIDDEN) {
    for (int l = 0; l < c->n_layers; ++l)
      o->hidden_in[l] = take((size_t)st->total[st->stage_of_layer[l]] * d * 2);
    o->hidden_out = take((size_t)st->total[st->stage_of_layer[c->n_layers - 1]] * d * 2);
  }
  o->total = off;
}

}  // namespace

namespace lz {
void set_last_hip_error(int e) { g_last_hip_error = e; }
}  // namespace lz

struct lazyllm_model {
  lazyllm_config cfg;
  int f_pad;
  char* blob;                                   // one device allocation holding everything below
  const void *embed, *final_norm, *lm_head;
  std::vector<const void*> attn_norm, ffn_norm, wqkv, wo, wgu, wdown;
  // 8-bit variant (cfg.gemm_dtype == 1): E4M3 codes of the same four matrices and one scale per row
  // the same four matrices in the layout of the decoding steps' weight-streaming kernel
  std::vector<const void*> wqkv_s, wo_s, wgu_s, wdown_s;
  std::vector<const void*> wqkv8, wo8, wgu8, wdown8;
  std::vector<const float*> sqkv, so, sgu, sdown;
};

extern "C" {

int lazyllm_abi_version(void) { return 3; }

const char* lazyllm_strerror(int status) {
  switch (status) {
    case LAZYLLM_OK: return "ok";
    case LAZYLLM_EINVAL: return "invalid argument";
    case LAZYLLM_ENOSPC: return "workspace or output buffer too small";
    case LAZYLLM_EHIP: return "HIP runtime failure";
    case LAZYLLM_ENOMEM: return "allocation failed";
    case LAZYLLM_EFAILED: return "generation handle unusable: an earlier decoding step failed part-way";
    default: return "unknown status";
  }
}

int lazyllm_last_hip_error(void) { return g_last_hip_error; }

int lazyllm_keep_counts(int32_t n, int32_t n_layers, const lazyllm_keep* sched, int32_t n_sched,
                        int32_t* n_per_layer) {
  if (n <= 0 || n_layers < 1 || n_layers > LAZYLLM_MAX_LAYERS || n_per_layer == nullptr)
    return LAZYLLM_EINVAL;
  if (!schedule_ok(n_layers, sched, n_sched)) return LAZYLLM_EINVAL;
  int m = n, i = 0;
  for (int l = 0; l < n_layers; ++l) {
    if (i < n_sched && sched[i].layer == l) { m = keep_count(m, sched[i].keep_permille); ++i; }
    n_per_layer[l] = m;
  }
  return LAZYLLM_OK;
}

size_t lazyllm_workspace_bytes(const lazyllm_config* cfg, int32_t total_tokens, int32_t batch,
                               int32_t max_seqlen) {
  if (!config_ok(cfg) || total_tokens <= 0 || batch <= 0 || max_seqlen <= 0 ||
      max_seqlen > total_tokens || batch > total_tokens)
    return 0;
  Workspace w;
  layout_workspace(cfg, total_tokens, batch, max_seqlen, &w);
  return w.total;
}

size_t lazyllm_output_bytes(const lazyllm_config* cfg, const int32_t* seqlens, int32_t batch,
                            const lazyllm_keep* sched, int32_t n_sched, uint32_t flags) {
  if (!config_ok(cfg) || seqlens == nullptr || batch <= 0 || (flags & ~7u) != 0) return 0;
  if (!schedule_ok(cfg->n_layers, sched, n_sched)) return 0;
  long long total = 0;
  for (int b = 0; b < batch; ++b) {
    if (seqlens[b] <= 0) return 0;
    total += seqlens[b];
  }
  if (total > 0x7fffffffLL / 4) return 0;
  Stages st;
  build_stages(cfg->n_layers, sched, n_sched, seqlens, batch, &st);
  Output o;
  layout_output(cfg, &st, batch, flags, &o);
  return o.total;
}

// ---- model --------------------------------------------------------------------------------

int lazyllm_model_create(const lazyllm_config* cfg, const lazyllm_weights* w, void* hip_stream,
                         lazyllm_model** out) {
  if (!config_ok(cfg) || w == nullptr || out == nullptr) return LAZYLLM_EINVAL;
  if (!w->embed || !w->attn_norm || !w->wq || !w->wk || !w->wv || !w->wo || !w->ffn_norm ||
      !w->w_gate || !w->w_up || !w->w_down || !w->final_norm || !w->lm_head)
    return LAZYLLM_EINVAL;
  const int L = cfg->n_layers;
  for (int l = 0; l < L; ++l)
    if (!w->attn_norm[l] || !w->wq[l] || !w->wk[l] || !w->wv[l] || !w->wo[l] || !w->ffn_norm[l] ||
        !w->w_gate[l] || !w->w_up[l] || !w->w_down[l])
      return LAZYLLM_EINVAL;

  lazyllm_model* m = new (std::nothrow) lazyllm_model();
  if (m == nullptr) return LAZYLLM_ENOMEM;
  m->cfg = *cfg;
  m->f_pad = ffn_padded(cfg->d_ffn);
  const size_t d = cfg->d_model, f = cfg->d_ffn, fp = m->f_pad, V = cfg->vocab, kvd = kv_dim(cfg);
  const size_t per_layer = align_up(d * 2) * 2 + 2 * (align_up((d + 2 * kvd) * d * 2) + align_up(d * d * 2) +
                                                      align_up(2 * fp * d * 2) + align_up(d * fp * 2));
  const bool f8 = cfg->gemm_dtype == 1;
  const size_t per_layer8 = !f8 ? 0 : align_up((d + 2 * kvd) * d) + align_up(d * d) + align_up(2 * fp * d) +
                                          align_up(d * fp) + align_up((d + 2 * kvd) * 4) + 2 * align_up(d * 4) +
                                          align_up(2 * fp * 4);
  const size_t bytes = align_up(V * d * 2) * 2 + align_up(d * 2) + (per_layer + per_layer8) * L;
  hipError_t e = hipMalloc((void**)&m->blob, bytes);
  if (e != hipSuccess) {
    delete m;
    g_last_hip_error = (int)e;
    return e == hipErrorOutOfMemory ? LAZYLLM_ENOMEM : LAZYLLM_EHIP;
  }
  hipStream_t st = (hipStream_t)hip_stream;
  size_t off = 0;
  auto take = [&](size_t b) { char* p = m->blob + off; off += align_up(b); return p; };
  int rc = LAZYLLM_OK;
  auto chk = [&](hipError_t err) { if (err != hipSuccess && rc == LAZYLLM_OK) rc = hip_fail(err); };

  char* p = take(V * d * 2);
  chk(hipMemcpyAsync(p, w->embed, V * d * 2, hipMemcpyDeviceToDevice, st));
  m->embed = p;
  p = take(V * d * 2);
  chk(hipMemcpyAsync(p, w->lm_head, V * d * 2, hipMemcpyDeviceToDevice, st));
  m->lm_head = p;
  p = take(d * 2);
  chk(hipMemcpyAsync(p, w->final_norm, d * 2, hipMemcpyDeviceToDevice, st));
  m->final_norm = p;
  // The four matrices of a layer are first put together row-major in a staging buffer (fused,
  // gains folded in, padded) and then stored in the forms the kernels read: K-step-major for the
  // tile kernels, sequential streams for the decoding steps' weight-streaming kernel, and, for the
  // 8-bit variant, E4M3 codes with row scales.  The staging buffer is reused layer after layer
  // (everything runs in order on one stream) and freed at the end.
  const size_t n_qkv = (d + 2 * kvd) * d * 2, n_o = d * d * 2, n_gu = 2 * fp * d * 2, n_down = d * fp * 2;
  char* staging = nullptr;
  const size_t n_codes = f8 ? std::max(std::max(n_qkv, n_o), std::max(n_gu, n_down)) / 2 : 0;
  e = hipMalloc((void**)&staging, align_up(n_qkv) + align_up(n_o) + align_up(n_gu) + align_up(n_down) +
                                      align_up(n_codes));
  if (e != hipSuccess) {
    (void)hipFree(m->blob);
    delete m;
    g_last_hip_error = (int)e;
    return e == hipErrorOutOfMemory ? LAZYLLM_ENOMEM : LAZYLLM_EHIP;
  }
  char* t_qkv = staging;
  char* t_o = t_qkv + align_up(n_qkv);
  char* t_gu = t_o + align_up(n_o);
  char* t_down = t_gu + align_up(n_gu);
  char* t_codes = t_down + align_up(n_down);
  for (int l = 0; l < L && rc == LAZYLLM_OK; ++l) {
    p = take(d * 2);
    chk(hipMemcpyAsync(p, w->attn_norm[l], d * 2, hipMemcpyDeviceToDevice, st));
    m->attn_norm.push_back(p);
    p = take(d * 2);
    chk(hipMemcpyAsync(p, w->ffn_norm[l], d * 2, hipMemcpyDeviceToDevice, st));
    m->ffn_norm.push_back(p);
    // fused [q; k; v] rows
    chk(hipMemcpyAsync(t_qkv, w->wq[l], d * d * 2, hipMemcpyDeviceToDevice, st));
    chk(hipMemcpyAsync(t_qkv + d * d * 2, w->wk[l], kvd * d * 2, hipMemcpyDeviceToDevice, st));
    chk(hipMemcpyAsync(t_qkv + (d + kvd) * d * 2, w->wv[l], kvd * d * 2, hipMemcpyDeviceToDevice, st));
    // RMSNorm gains ride in the weights: x*g . w = x . (g*w); the 1/rms factor is applied by the
    // GEMM epilogue (exact for gains of 1, one more bf16 rounding of the weight otherwise)
    chk(launch_scale_cols(t_qkv, w->attn_norm[l], d + 2 * kvd, (int)d, st));
    chk(hipMemcpyAsync(t_o, w->wo[l], d * d * 2, hipMemcpyDeviceToDevice, st));
    // gate/up interleaved in 32-row blocks
    chk(launch_interleave_gate_up(w->w_gate[l], w->w_up[l], t_gu, (int)f, (int)fp, (int)d, st));
    chk(launch_scale_cols(t_gu, w->ffn_norm[l], 2 * fp, (int)d, st));
    // down, K zero-padded to f_pad
    chk(launch_copy_rows(w->w_down[l], t_down, (int)d, (int)f, (int)f, (int)fp, st));
    auto store = [&](const char* src, size_t rows, size_t K, std::vector<const void*>& tiles,
                     std::vector<const void*>& streams, std::vector<const void*>& codes,
                     std::vector<const float*>& scales) {
      char* pb = take(rows * K * 2);
      chk(launch_pack_kblock(src, (int)rows, (int)K, (int)K, pb, st));
      tiles.push_back(pb);
      char* ps = take(rows * K * 2);
      chk(launch_pack_stream(src, (int)rows, (int)K, (int)K, ps, st));
      streams.push_back(ps);
      if (f8) {
        // codes row by row into the staging buffer, then K-step-major like the 16-bit form
        // (a row of K codes = K / 2 16-bit units: the same rearrangement in 128-byte pieces)
        char* c8 = take(rows * K);
        float* sc = (float*)take(rows * 4);
        chk(launch_quantize_rows_f8(src, (int)rows, (int)K, (int)K, t_codes, (int)K, sc, st));
        chk(launch_pack_kblock(t_codes, (int)rows, (int)(K / 2), (int)(K / 2), c8, st));
        codes.push_back(c8);
        scales.push_back(sc);
      }
    };
    store(t_qkv, d + 2 * kvd, d, m->wqkv, m->wqkv_s, m->wqkv8, m->sqkv);
    store(t_o, d, d, m->wo, m->wo_s, m->wo8, m->so);
    store(t_gu, 2 * fp, d, m->wgu, m->wgu_s, m->wgu8, m->sgu);
    store(t_down, d, fp, m->wdown, m->wdown_s, m->wdown8, m->sdown);
  }
  if (rc == LAZYLLM_OK) chk(hipStreamSynchronize(st));
  else (void)hipStreamSynchronize(st);
  (void)hipFree(staging);
  if (rc != LAZYLLM_OK) {
    (void)hipFree(m->blob);
    delete m;
    return rc;
  }
  *out = m;
  return LAZYLLM_OK;
}

void lazyllm_model_destroy(lazyllm_model* m) {
  if (m == nullptr) return;
  (void)hipFree(m->blob);
  delete m;
}

// ---- prefill ------------------------------------------------------------------------------

int lazyllm_prefill_varlen(const lazyllm_model* m, const int32_t* token_ids,
                           const float* embed_scale, const int32_t* cu_host,
                           const int32_t* cu_dev, int32_t batch, const lazyllm_keep* sched,
                           int32_t n_sched, uint32_t flags, void* workspace, size_t ws_bytes,
                           void* out_buf, size_t out_bytes, void* hip_stream, lazyllm_result* res) {
  // ---- validation: nothing below this block is reached with a bad argument, and nothing in
  // this block touches HIP
  if (m == nullptr || token_ids == nullptr || cu_host == nullptr || workspace == nullptr ||
      out_buf == nullptr || res == nullptr || batch <= 0)
    return LAZYLLM_EINVAL;
  if (batch > 1 && cu_dev == nullptr) return LAZYLLM_EINVAL;
  if ((flags & ~7u) != 0) return LAZYLLM_EINVAL;
  if (((uintptr_t)workspace & 255) != 0 || ((uintptr_t)out_buf & 255) != 0) return LAZYLLM_EINVAL;
  const lazyllm_config* c = &m->cfg;
  if (!schedule_ok(c->n_layers, sched, n_sched)) return LAZYLLM_EINVAL;
  if (cu_host[0] != 0) return LAZYLLM_EINVAL;
  std::vector<int32_t> seqlens(batch);
  int max_seqlen = 0;
  for (int b = 0; b < batch; ++b) {
    const long long n = (long long)cu_host[b + 1] - cu_host[b];
    if (n <= 0 || cu_host[b + 1] > 0x7fffffff / 4) return LAZYLLM_EINVAL;
    seqlens[b] = (int32_t)n;
    if (n > max_seqlen) max_seqlen = (int)n;
  }
  const int T = cu_host[batch];
  Stages stg;
  build_stages(c->n_layers, sched, n_sched, seqlens.data(), batch, &stg);
  Workspace ws;
  layout_workspace(c, T, batch, max_seqlen, &ws);
  Output ob;
  layout_output(c, &stg, batch, flags, &ob);
  if (ws_bytes < ws.total || out_bytes < ob.total) return LAZYLLM_ENOSPC;

  // ---- result struct
  char* W = (char*)workspace;
  char* O = (char*)out_buf;
  const int L = c->n_layers, d = c->d_model, H = c->n_heads, hd = c->head_dim, B = batch;
  const int kvd = kv_dim(c), kv_group = H / kv_heads(c);
  const int BW = B + 1;
  memset(res, 0, sizeof(*res));
  res->batch = B;
  res->n_layers = L;
  res->logits = (float*)(O + ob.logits);
  res->status = (int32_t*)(O + ob.status);
  int32_t* cu_stage = (int32_t*)(O + ob.cu_stage);
  int32_t* cu_aux = (int32_t*)(O + ob.cu_aux);
  int32_t* cu_vt = (int32_t*)(O + ob.cu_vt);
  const bool score_all = (flags & LAZYLLM_SCORE_ONLY_USED) == 0;
  for (int l = 0; l < L; ++l) {
    const int s = stg.stage_of_layer[l];
    res->n_tokens[l] = (int32_t)stg.total[s];
    res->kept_pos[l] = (int32_t*)(O + ob.kept_pos[s]);
    res->cu_kept[l] = cu_stage + s * BW;
    res->k[l] = O + ob.k[l];
    res->v[l] = O + ob.v[l];
    const bool used = (l + 1 < L) && stg.stage_of_layer[l + 1] != s;
    res->scores[l] = (score_all || used) ? (float*)(O + ob.scores[l]) : nullptr;
    if (s > 0 && stg.first_layer[s] == l) {
      res->n_aux[l] = (int32_t)(stg.total[s - 1] - stg.total[s]);
      res->aux_h[l] = O + ob.aux_h[s];
      res->aux_pos[l] = (int32_t*)(O + ob.aux_pos[s]);
      res->cu_aux[l] = cu_aux + (s - 1) * BW;
    }
  }

  // ---- enqueue
  hipStream_t st = (hipStream_t)hip_stream;
  PlanArgs plan;
  memset(&plan, 0, sizeof(plan));
  plan.n_stages = stg.n_stages - 1;
  for (int s = 1; s < stg.n_stages; ++s) plan.permille[s - 1] = stg.permille[s];
  const double dd = (double)d, rowb = dd * 2.0;      // bytes of one bf16 row
  // tickets and flags of the GEMM forms that exchange partial tiles between workgroups
  LZ_HIP(launch_gemm_counters_clear(W + ws.gemm_ws, st));
  LZ_RUN(LAZYLLM_STEP_PLAN, -1, T, 0.0,
         launch_plan(cu_dev, seqlens.data(), B, T, plan, cu_stage, cu_aux, cu_vt, res->status, st));
  float2* rope = (float2*)(W + ws.rope);
  LZ_RUN(LAZYLLM_STEP_ROPE_TABLE, -1, max_seqlen, (double)max_seqlen * (hd / 2) * 8.0,
         launch_rope_table(rope, max_seqlen, hd, c->rope_theta, st));
  char* hbuf[2] = {W + ws.h0, W + ws.h1};
  int cur = 0;
  LZ_RUN(LAZYLLM_STEP_EMBED, -1, T, 2.0 * T * rowb,
         launch_embed(m->embed, token_ids, embed_scale, cu_stage, B, T, d, c->vocab, hbuf[0],
                      res->kept_pos[0], res->status, st, (unsigned long long*)(W + ws.ssq0)));
  const int fp = m->f_pad;
  // RMSNorm is folded into the projections that consume it (no launch, no normalised copy of
  // h): whoever writes h also leaves each row's sum of squares -- the embedding and compaction
  // kernels directly, the two residual GEMMs by integer atomics from their epilogues -- and the
  // QKV and gate/up GEMMs scale their output rows by 1/rms (gains are folded into their weights).
  // ssq_attn belongs to the h that enters a layer, ssq_ffn to the h after the attention block;
  // each is zeroed by the GEMM that runs just before the one that accumulates into it.
  unsigned long long* ssq_attn = (unsigned long long*)(W + ws.ssq0);
  unsigned long long* ssq_ffn = (unsigned long long*)(W + ws.ssq1);
  const float ssq_mul = 1.0f / (4294967296.0f * (float)d);
  // Compaction folded into the operand loads of the layer that follows a selection: not with the
  // 8-bit projections (their row quantiser reads A itself) nor when the caller wants every layer's
  // input rows copied out.
  const bool fuse_compaction = (flags & LAZYLLM_FUSE_COMPACTION) != 0 && c->gemm_dtype == 0 &&
                               (flags & LAZYLLM_KEEP_HIDDEN) == 0;
  for (int l = 0; l < L; ++l) {
    const int s = stg.stage_of_layer[l];
    const int n = (int)stg.total[s];
    const int32_t* cu = cu_stage + s * BW;
    const int32_t* rows_of_h = nullptr;             // set: row t of this layer's input is row rows_of_h[t] of h
    if (s > 0 && stg.first_layer[s] == l) {
      // Sec. 3.2: the scores of layer l-1 pick the tokens that enter layer l; the others'
      // hidden states go to this layer's Aux Cache.
      const int n_prev = (int)stg.total[s - 1];
      int32_t* keep_idx = (int32_t*)(W + ws.keep_idx);
      int32_t* prune_idx = (int32_t*)(W + ws.prune_idx);
      LZ_RUN(LAZYLLM_STEP_SELECT, l, n_prev, 8.0 * n_prev,
             launch_select(res->scores[l - 1], cu_stage + (s - 1) * BW, cu, 0, 0, B, keep_idx,
                           prune_idx, st));
      if (fuse_compaction) {
        // only the dropped rows move (to the Aux Cache) and the positions are compacted; the kept
        // rows stay where they are (read once, for the same sums of squares as the copying form
        // leaves) and this layer's QKV projection (A operand, row scales) and O projection
        // (residual) read them through keep_idx, the O projection writing the compact hidden
        // states into the other buffer
        LZ_RUN(LAZYLLM_STEP_GATHER, l, n_prev, 2.0 * (n_prev - n) * rowb,
               launch_gather(hbuf[cur], res->kept_pos[l - 1], keep_idx, n, prune_idx, n_prev - n,
                             nullptr, res->kept_pos[l], res->aux_h[l], res->aux_pos[l], d, st,
                             ssq_attn));
        rows_of_h = keep_idx;
      } else {
        LZ_RUN(LAZYLLM_STEP_GATHER, l, n_prev, 2.0 * n_prev * rowb,
               launch_gather(hbuf[cur], res->kept_pos[l - 1], keep_idx, n, prune_idx, n_prev - n,
                             hbuf[cur ^ 1], res->kept_pos[l], res->aux_h[l], res->aux_pos[l], d, st,
                             ssq_attn));
        cur ^= 1;
      }
    }
    char* h = hbuf[cur];                            // the layer's input (rows through rows_of_h, if set)
    // One projection: the 16-bit GEMM, or in the 8-bit variant the row quantiser on the operand
    // followed by the 8-bit GEMM with the same epilogue (both in the step's timing).
    auto project = [&](const void* A, int K, const void* w16, const void* w8, const float* sw8,
                       void* Cout, const void* R, int N, int ldc, int epi, const EpiArgs* ea,
                       bool stream_k) -> hipError_t {
      if (c->gemm_dtype == 0) {
        EpiArgs eb = *ea;
        eb.w_blocked = 1;                            // the model's 16-bit weights are K-step-major
        eb.psk_ready = 1;                            // (flags cleared at the start of this call)
        (void)stream_k;
        return launch_gemm(A, w16, Cout, R, n, N, K, K, K, ldc, epi, st, &eb, W + ws.gemm_ws,
                           gemm_workspace_bytes());
      }
      hipError_t qe = launch_quantize_rows_f8(A, n, K, K, W + ws.a8, K, (float*)(W + ws.sa8), st);
      if (qe != hipSuccess) return qe;
      EpiArgs e8 = *ea;
      e8.w_blocked = 1;                              // the model's codes are K-step-major too
      return launch_gemm_f8(W + ws.a8, (const float*)(W + ws.sa8), w8, sw8, Cout, R, n, N, K, K, K, ldc,
                            epi, st, &e8);
    };
    const bool f8 = c->gemm_dtype == 1;
    if (flags & LAZYLLM_KEEP_HIDDEN) {
      res->hidden_in[l] = O + ob.hidden_in[l];
      LZ_HIP(hipMemcpyAsync(res->hidden_in[l], h, (size_t)n * d * 2, hipMemcpyDeviceToDevice, st));
    }
    // causal attention: 2 products of 2*hd FLOPs per (query, visible key, head)
    double att_flops = 0.0;
    for (int b = 0; b < B; ++b) {
      int nb = seqlens[b];
      for (int k = 1; k <= s; ++k) nb = keep_count(nb, stg.permille[k]);
      att_flops += 2.0 * (double)nb * ((double)nb + 1.0) * dd;
    }
    // QKV projection with the rotary embedding (original positions) applied in the epilogue;
    // K and V land directly in this layer's KV cache.
    EpiArgs ra{};
    ra.pos = res->kept_pos[l]; ra.table = rope;
    ra.q = (uint16_t*)(W + ws.q); ra.k = (uint16_t*)res->k[l]; ra.v = (uint16_t*)res->v[l];
    ra.d_model = d; ra.head_dim = hd; ra.kv_dim = kvd;
    // ... and V also transposed into the workspace copy the attention kernel reads
    ra.vt = (uint16_t*)(W + ws.vt); ra.vt_ld = (int)stg.vt_ld[s];
    ra.vt_col = B > 1 ? (const int32_t*)(W + ws.vt_col) : nullptr;
    ra.ssq_in = ssq_attn; ra.ssq_mul = ssq_mul; ra.eps = c->rms_eps; ra.ssq_clear = ssq_ffn;
    ra.a_rows = rows_of_h;
    if (stg.first_layer[s] == l)
      LZ_RUN(LAZYLLM_STEP_V_TRANSPOSE, l, n, 0.0,
             launch_vt_stage_setup(W + ws.vt, B > 1 ? (int32_t*)(W + ws.vt_col) : nullptr, cu,
                                   cu_vt + s * BW, 0, B, (int)stg.vt_ld[s], kvd, st));
    LZ_RUN(LAZYLLM_STEP_GEMM_QKV, l, n, 2.0 * n * (dd + 2.0 * kvd) * dd,
           project(h, d, m->wqkv[l], f8 ? m->wqkv8[l] : nullptr, f8 ? m->sqkv[l] : nullptr, nullptr,
                   nullptr, d + 2 * kvd, 0, EPI_QKV_ROPE, &ra, false));
    // Eq. 1 needs the last query's logits against every key, which the attention kernel has
    // in registers anyway: it leaves them in the score scratch (the gate/up launch below turns
    // them into the head-averaged probabilities).
    const bool scored = res->scores[l] != nullptr;
    LZ_RUN(LAZYLLM_STEP_ATTENTION, l, n, att_flops,
           launch_attention(W + ws.q, res->k[l], W + ws.vt, W + ws.o, cu, cu_vt + s * BW, 0, B,
                            stg.max_rows[s], (int)stg.vt_ld[s], H, hd, st,
                            scored ? score_z(W + ws.score) : nullptr,
                            scored ? score_zstat(W + ws.score, (int)stg.vt_ld[s], H) : nullptr,
                            (int)stg.vt_ld[s], kv_group));
    EpiArgs eo{};
    eo.ssq_out = ssq_ffn;
    eo.r_rows = rows_of_h;
    if (rows_of_h != nullptr) {                     // residual rows through the index, output compact
      LZ_RUN(LAZYLLM_STEP_GEMM_O, l, n, 2.0 * n * dd * dd,
             project(W + ws.o, d, m->wo[l], nullptr, nullptr, hbuf[cur ^ 1], h, d, d, EPI_RESIDUAL, &eo, true));
      cur ^= 1;
      h = hbuf[cur];
    } else {
      LZ_RUN(LAZYLLM_STEP_GEMM_O, l, n, 2.0 * n * dd * dd,
             project(W + ws.o, d, m->wo[l], f8 ? m->wo8[l] : nullptr, f8 ? m->so[l] : nullptr, h, h, d, d,
                     EPI_RESIDUAL, &eo, true));
    }
    EpiArgs eg{};
    eg.ssq_in = ssq_ffn; eg.ssq_mul = ssq_mul; eg.eps = c->rms_eps; eg.ssq_clear = ssq_attn;
    if (scored) {
      // Eq. 1's last step (softmax of the logits the attention kernel left, averaged over heads)
      // rides in this launch as extra workgroups behind the GEMM's tiles
      eg.sf_z = score_z(W + ws.score);
      eg.sf_stat = (const float2*)score_zstat(W + ws.score, (int)stg.vt_ld[s], H);
      eg.sf_s = res->scores[l];
      eg.sf_cu = cu; eg.sf_cu_z = cu_vt + s * BW;
      eg.sf_n_single = 0; eg.sf_heads = H; eg.sf_z_ld = (int)stg.vt_ld[s];
      eg.sf_max_rows = stg.max_rows[s]; eg.sf_batch = B;
    }
    LZ_RUN(LAZYLLM_STEP_GEMM_GATE_UP, l, n, 2.0 * n * 2.0 * (double)c->d_ffn * dd,
           project(h, d, m->wgu[l], f8 ? m->wgu8[l] : nullptr, f8 ? m->sgu[l] : nullptr, W + ws.act,
                   nullptr, 2 * fp, fp, EPI_SWIGLU, &eg, false));
    EpiArgs ed{};
    ed.ssq_out = ssq_attn;
    LZ_RUN(LAZYLLM_STEP_GEMM_DOWN, l, n, 2.0 * n * (double)c->d_ffn * dd,
           project(W + ws.act, fp, m->wdown[l], f8 ? m->wdown8[l] : nullptr, f8 ? m->sdown[l] : nullptr,
                   h, h, d, d, EPI_RESIDUAL, &ed, true));
  }
  const int s_last = stg.stage_of_layer[L - 1];
  if (flags & LAZYLLM_KEEP_HIDDEN) {
    res->hidden_out = O + ob.hidden_out;
    LZ_HIP(hipMemcpyAsync(res->hidden_out, hbuf[cur], (size_t)stg.total[s_last] * d * 2,
                          hipMemcpyDeviceToDevice, st));
  }
  LZ_HIP(launch_gemm_exchange_check(W + ws.gemm_ws, res->status, st));
  if (lm_head_fused_fits(B, d)) {
    LZ_RUN(LAZYLLM_STEP_LM_HEAD, -1, B, (double)c->vocab * rowb,
           launch_lm_head_fused(hbuf[cur], cu_stage + s_last * BW, 0, B, m->final_norm, m->lm_head,
                                res->logits, d, c->vocab, c->rms_eps, st));
  } else {
    LZ_RUN(LAZYLLM_STEP_LM_HEAD, -1, B, (double)c->vocab * rowb,
           launch_final_norm(hbuf[cur], cu_stage + s_last * BW, 0, B, m->final_norm,
                             (float*)(W + ws.xf), d, c->rms_eps, st));
    LZ_RUN(LAZYLLM_STEP_LM_HEAD, -1, B, 0.0,
           launch_lm_head((const float*)(W + ws.xf), m->lm_head, res->logits, B, d, c->vocab, st));
  }
  return LAZYLLM_OK;
}

int lazyllm_prefill(const lazyllm_model* m, const int32_t* token_ids, const float* embed_scale,
                    int32_t n, const lazyllm_keep* sched, int32_t n_sched, uint32_t flags,
                    void* workspace, size_t ws_bytes, void* out_buf, size_t out_bytes,
                    void* hip_stream, lazyllm_result* res) {
  if (n <= 0) return LAZYLLM_EINVAL;
  const int32_t cu[2] = {0, n};
  return lazyllm_prefill_varlen(m, token_ids, embed_scale, cu, nullptr, 1, sched, n_sched, flags,
                                workspace, ws_bytes, out_buf, out_bytes, hip_stream, res);
}

// ---- decoding steps with the Aux Cache (Sec. 3.2) ------------------------------------------

}  // extern "C"

namespace {

static_assert(ST_BAD_TOKEN == LAZYLLM_ST_BAD_TOKEN && ST_BAD_CU == LAZYLLM_ST_BAD_CU &&
              ST_NO_STATE == LAZYLLM_ST_NO_STATE && ST_EXCHANGE == LAZYLLM_ST_EXCHANGE, "status bits");

inline int round_up64(int x) { return (x + 63) / 64 * 64; }

// Generation state inside the caller's buffer (offsets), everything indexed by position.
struct GenLayout {
  size_t k[LAZYLLM_MAX_LAYERS], vt[LAZYLLM_MAX_LAYERS];
  size_t has_kv[LAZYLLM_MAX_LAYERS + 1], aux_h[LAZYLLM_MAX_LAYERS + 1], has_aux[LAZYLLM_MAX_LAYERS + 1];
  size_t rope, status, logits, total;
  int vt_ld;
};

void layout_generation(const lazyllm_config* c, const Stages* st, int cap, GenLayout* g) {
  const size_t d = c->d_model;
  g->vt_ld = round_up64(cap);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t r = off; off += align_up(bytes); return r; };
  g->status = take(4);
  g->logits = take((size_t)c->vocab * 4);
  g->rope = take((size_t)cap * (c->head_dim / 2) * sizeof(float2));
  for (int s = 0; s < st->n_stages; ++s) {
    g->has_kv[s] = take((size_t)cap);
    g->has_aux[s] = take((size_t)cap);
    g->aux_h[s] = s > 0 ? take((size_t)cap * d * 2) : 0;
  }
  for (int l = 0; l < c->n_layers; ++l) {
    g->k[l] = take((size_t)cap * kv_dim(c) * 2);
    g->vt[l] = take((size_t)kv_dim(c) * g->vt_ld * 2);
  }
  g->total = off;
}

// Scratch of one step; rows are bounded by the capacity (every token could be revived at once).
struct GenWorkspace {
  size_t h0, h1, ssq0, ssq1, q, o, act, score, scores, member, bits, run_pos, live_row, src_row,
      park_src, park_pos, counts, xf, att_ws, gemm_ws, total;
};

void layout_gen_workspace(const lazyllm_config* c, int n_stages, int cap, GenWorkspace* w) {
  const size_t d = c->d_model, fp = ffn_padded(c->d_ffn), T = (size_t)cap;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
  w->h0 = take(T * d * 2);
  w->h1 = take(T * d * 2);
  w->ssq0 = take(T * 8);
  w->ssq1 = take(T * 8);
  w->q = take(T * d * 2);
  w->o = take(T * d * 2);
  w->act = take(T * fp * 2);
  w->score = take(score_scratch_bytes(cap, 1, c->n_heads));
  w->scores = take((size_t)c->n_layers * T * 4);
  w->member = take((size_t)n_stages * T);
  w->bits = take((size_t)n_stages * (round_up64(cap) / 64) * 8);
  w->run_pos = take((size_t)n_stages * T * 4);
  w->live_row = take(T * 4);
  w->src_row = take(T * 4);
  w->park_src = take(T * 4);
  w->park_pos = take(T * 4);
  w->counts = take((size_t)n_stages * 16);
  w->xf = take(d * 4);
  w->att_ws = take(decode_attention_workspace_bytes(c->d_model, c->n_heads));
  w->gemm_ws = take(gemm_workspace_bytes());
  w->total = off;
}

}  // namespace

struct lazyllm_generation {
  const lazyllm_model* m;
  Stages stg;               // stage table of the schedule (token counts are per step)
  GenLayout gl;
  char* state;
  int capacity, n_prompt, n_tokens;
  int32_t* host_counts;     // pinned host memory, [n_stages][4]
  // set while a step is being enqueued and cleared when it has been enqueued completely: a step
  // that returns an error after its first launch has already changed has_kv / has_aux / live_row
  // without advancing n_tokens, so every later step is refused
  bool failed;
};

extern "C" {

size_t lazyllm_generation_state_bytes(const lazyllm_config* cfg, const lazyllm_keep* sched,
                                      int32_t n_sched, int32_t capacity) {
  if (!config_ok(cfg) || capacity <= 0 || capacity > 0x7fffffff / 8) return 0;
  if (!schedule_ok(cfg->n_layers, sched, n_sched)) return 0;
  Stages st;
  const int32_t one = 1;
  build_stages(cfg->n_layers, sched, n_sched, &one, 1, &st);
  GenLayout g;
  layout_generation(cfg, &st, capacity, &g);
  return g.total;
}

size_t lazyllm_decode_workspace_bytes(const lazyllm_config* cfg, const lazyllm_keep* sched,
                                      int32_t n_sched, int32_t capacity) {
  if (!config_ok(cfg) || capacity <= 0 || capacity > 0x7fffffff / 8) return 0;
  if (!schedule_ok(cfg->n_layers, sched, n_sched)) return 0;
  Stages st;
  const int32_t one = 1;
  build_stages(cfg->n_layers, sched, n_sched, &one, 1, &st);
  GenWorkspace w;
  layout_gen_workspace(cfg, st.n_stages, capacity, &w);
  return w.total;
}

int lazyllm_generation_create(const lazyllm_model* m, const lazyllm_keep* sched, int32_t n_sched,
                              int32_t capacity, const lazyllm_result* prefill, void* state,
                              size_t state_bytes, void* hip_stream, lazyllm_generation** out) {
  if (m == nullptr || prefill == nullptr || state == nullptr || out == nullptr) return LAZYLLM_EINVAL;
  if (((uintptr_t)state & 255) != 0) return LAZYLLM_EINVAL;
  const lazyllm_config* c = &m->cfg;
  if (!schedule_ok(c->n_layers, sched, n_sched)) return LAZYLLM_EINVAL;
  if (prefill->batch != 1 || prefill->n_layers != c->n_layers) return LAZYLLM_EINVAL;
  const int n_prompt = prefill->n_tokens[0];
  if (n_prompt <= 0 || capacity <= n_prompt || capacity > 0x7fffffff / 8) return LAZYLLM_EINVAL;
  Stages stg;
  build_stages(c->n_layers, sched, n_sched, &n_prompt, 1, &stg);
  for (int l = 0; l < c->n_layers; ++l) {          // the prefill must be one made with this schedule
    const int s = stg.stage_of_layer[l];
    if (prefill->n_tokens[l] != (int32_t)stg.total[s] || prefill->kept_pos[l] == nullptr ||
        prefill->k[l] == nullptr || prefill->v[l] == nullptr)
      return LAZYLLM_EINVAL;
    if (s > 0 && stg.first_layer[s] == l &&
        (prefill->n_aux[l] != (int32_t)(stg.total[s - 1] - stg.total[s]) ||
         (prefill->n_aux[l] > 0 && (prefill->aux_h[l] == nullptr || prefill->aux_pos[l] == nullptr))))
      return LAZYLLM_EINVAL;
  }
  GenLayout gl;
  layout_generation(c, &stg, capacity, &gl);
  if (state_bytes < gl.total) return LAZYLLM_ENOSPC;

  lazyllm_generation* g = new (std::nothrow) lazyllm_generation();
  if (g == nullptr) return LAZYLLM_ENOMEM;
  g->m = m; g->stg = stg; g->gl = gl; g->state = (char*)state;
  g->capacity = capacity; g->n_prompt = n_prompt; g->n_tokens = n_prompt; g->failed = false;
  g->host_counts = nullptr;
  hipError_t e = hipHostMalloc((void**)&g->host_counts, (size_t)stg.n_stages * 16, hipHostMallocDefault);
  if (e != hipSuccess) {
    delete g;
    g_last_hip_error = (int)e;
    return LAZYLLM_ENOMEM;
  }
  hipStream_t st = (hipStream_t)hip_stream;
  int rc = LAZYLLM_OK;
  auto chk = [&](hipError_t err) { if (err != hipSuccess && rc == LAZYLLM_OK) rc = hip_fail(err); };
  char* S = g->state;
  const int d = c->d_model;
  // entries never written must still be finite: the attention kernel multiplies the V of
  // masked keys by probabilities that are exactly 0
  chk(launch_fill_zero(S, gl.total, st));
  chk(launch_rope_table((float2*)(S + gl.rope), capacity, c->head_dim, c->rope_theta, st));
  for (int l = 0; l < c->n_layers && rc == LAZYLLM_OK; ++l) {
    const int s = stg.stage_of_layer[l];
    const int n = prefill->n_tokens[l];
    chk(launch_scatter_rows(prefill->k[l], prefill->kept_pos[l], n, S + gl.k[l],
                            stg.first_layer[s] == l ? (uint8_t*)(S + gl.has_kv[s]) : nullptr, kv_dim(c), st));
    chk(launch_scatter_vt(prefill->v[l], prefill->kept_pos[l], n, kv_dim(c), S + gl.vt[l], gl.vt_ld, st));
    if (s > 0 && stg.first_layer[s] == l)
      chk(launch_scatter_rows(prefill->aux_h[l], prefill->aux_pos[l], prefill->n_aux[l],
                              S + gl.aux_h[s], (uint8_t*)(S + gl.has_aux[s]), d, st));
  }
  if (rc != LAZYLLM_OK) {
    (void)hipHostFree(g->host_counts);
    delete g;
    return rc;
  }
  *out = g;
  return LAZYLLM_OK;
}

void lazyllm_generation_destroy(lazyllm_generation* g) {
  if (g == nullptr) return;
  if (g->host_counts != nullptr) (void)hipHostFree(g->host_counts);
  delete g;
}

int lazyllm_generation_get_view(const lazyllm_generation* g, lazyllm_generation_view* v) {
  if (g == nullptr || v == nullptr) return LAZYLLM_EINVAL;
  memset(v, 0, sizeof(*v));
  const lazyllm_config* c = &g->m->cfg;
  v->n_layers = c->n_layers; v->capacity = g->capacity; v->n_prompt = g->n_prompt;
  v->n_tokens = g->n_tokens; v->vt_ld = g->gl.vt_ld;
  char* S = g->state;
  for (int l = 0; l < c->n_layers; ++l) {
    const int s = g->stg.stage_of_layer[l];
    v->k[l] = S + g->gl.k[l];
    v->vt[l] = S + g->gl.vt[l];
    v->has_kv[l] = (uint8_t*)(S + g->gl.has_kv[s]);
    if (s > 0 && g->stg.first_layer[s] == l) {
      v->aux_h[l] = S + g->gl.aux_h[s];
      v->has_aux[l] = (uint8_t*)(S + g->gl.has_aux[s]);
    }
  }
  return LAZYLLM_OK;
}

int lazyllm_decode_step(lazyllm_generation* g, const int32_t* token_id, void* workspace,
                        size_t ws_bytes, void* hip_stream, lazyllm_step_result* res) {
  if (g == nullptr || token_id == nullptr || workspace == nullptr || res == nullptr)
    return LAZYLLM_EINVAL;
  if (((uintptr_t)workspace & 255) != 0) return LAZYLLM_EINVAL;
  if (g->failed) return LAZYLLM_EFAILED;
  if (g->n_tokens >= g->capacity) return LAZYLLM_ENOSPC;
  const lazyllm_model* m = g->m;
  const lazyllm_config* c = &m->cfg;
  const Stages& stg = g->stg;
  const int NS = stg.n_stages;
  GenWorkspace ws;
  layout_gen_workspace(c, NS, g->capacity, &ws);
  if (ws_bytes < ws.total) return LAZYLLM_ENOSPC;

  const int L = c->n_layers, d = c->d_model, H = c->n_heads, hd = c->head_dim, fp = m->f_pad;
  const int kvd = kv_dim(c), kv_group = H / kv_heads(c);
  const int cap = g->capacity, new_pos = g->n_tokens, n_tot = g->n_tokens + 1;
  const GenLayout& gl = g->gl;
  char* S = g->state;
  char* W = (char*)workspace;
  hipStream_t st = (hipStream_t)hip_stream;
  int sel_count[LAZYLLM_MAX_LAYERS + 1];
  sel_count[0] = n_tot;
  for (int s = 1; s < NS; ++s) sel_count[s] = keep_count(sel_count[s - 1], stg.permille[s]);

  memset(res, 0, sizeof(*res));
  res->n_layers = L; res->n_tokens = n_tot; res->position = new_pos;
  res->logits = (float*)(S + gl.logits);
  res->status = (int32_t*)(S + gl.status);

  int32_t* live_row = (int32_t*)(W + ws.live_row);
  int32_t* src_row = (int32_t*)(W + ws.src_row);
  int32_t* park_src = (int32_t*)(W + ws.park_src);
  int32_t* park_pos = (int32_t*)(W + ws.park_pos);
  auto run_pos_of = [&](int s) { return (int32_t*)(W + ws.run_pos) + (size_t)s * cap; };
  auto member_of = [&](int s) { return (uint8_t*)(W + ws.member) + (size_t)s * cap; };
  auto bits_of = [&](int s) { return (unsigned long long*)(W + ws.bits) + (size_t)s * (round_up64(cap) / 64); };
  auto scores_of = [&](int l) { return (float*)(W + ws.scores) + (size_t)l * cap; };
  const float2* rope = (const float2*)(S + gl.rope);
  unsigned long long* ssq_attn = (unsigned long long*)(W + ws.ssq0);
  unsigned long long* ssq_ffn = (unsigned long long*)(W + ws.ssq1);
  const float ssq_mul = 1.0f / (4294967296.0f * (float)d);
  const double dd = (double)d, rowb = dd * 2.0;
  const int z_ld = gl.vt_ld;
  char* hbuf[2] = {W + ws.h0, W + ws.h1};
  int cur = 0, M = 1;

  g->failed = true;                  // until the whole step is enqueued (cleared at the end)
  LZ_HIP(launch_gemm_counters_clear(W + ws.gemm_ws, st));
  LZ_HIP(launch_decode_attention_counters_clear(W + ws.att_ws, decode_attention_workspace_bytes(d, H), st));
  LZ_RUN(LAZYLLM_STEP_EMBED, -1, 1, 2.0 * rowb,
         launch_gen_embed(m->embed, token_id, c->vocab, d, new_pos, hbuf[0], ssq_attn, run_pos_of(0),
                          live_row, (uint8_t*)(S + gl.has_kv[0]), res->status, st));
  for (int l = 0; l < L; ++l) {
    const int s = stg.stage_of_layer[l];
    if (s > 0 && stg.first_layer[s] == l) {
      // Sec. 3.2: this step's scores of layer l-1 pick the tokens of layer l; selected tokens
      // without K,V here run the layer (from the state they carry, or revived from this layer's
      // Aux Cache), unselected tokens that carry a state leave it in the Aux Cache.
      int32_t* counts_dev = (int32_t*)(W + ws.counts) + 4 * s;
      LZ_RUN(LAZYLLM_STEP_SELECT, l, n_tot, 8.0 * n_tot,
             launch_gen_stage(scores_of(l - 1), s > 1 ? member_of(s - 1) : nullptr, n_tot, sel_count[s],
                              member_of(s), bits_of(s), (uint8_t*)(S + gl.has_kv[s]),
                              (uint8_t*)(S + gl.has_aux[s]), live_row, run_pos_of(s), src_row,
                              park_src, park_pos, counts_dev, res->status, st));
      // how many rows run this stage decides every launch shape below: the one place a step
      // waits for the GPU
      LZ_HIP(hipMemcpyAsync(g->host_counts + 4 * s, counts_dev, 16, hipMemcpyDeviceToHost, st));
      LZ_HIP(hipStreamSynchronize(st));
      const int rows = g->host_counts[4 * s], parked = g->host_counts[4 * s + 1];
      if (rows < 1 || rows > sel_count[s] || parked < 0 || parked > M ||
          g->host_counts[4 * s + 2] != sel_count[s])
        return hip_fail(hipErrorUnknown);
      LZ_RUN(LAZYLLM_STEP_GATHER, l, rows + parked, 2.0 * (rows + parked) * rowb,
             launch_revive_gather(hbuf[cur], S + gl.aux_h[s], run_pos_of(s), src_row, rows, park_src,
                                  park_pos, parked, hbuf[cur ^ 1], ssq_attn, d, st));
      cur ^= 1;
      M = rows;
    }
    char* h = hbuf[cur];
    const int32_t* rpos = run_pos_of(s);
    res->n_selected[l] = sel_count[s];
    res->n_ran[l] = M;
    res->selected[l] = s > 0 ? member_of(s) : nullptr;
    res->ran_pos[l] = rpos;
    res->scores[l] = scores_of(l);

    EpiArgs ra{};
    ra.pos = rpos; ra.table = rope;
    ra.q = (uint16_t*)(W + ws.q); ra.k = (uint16_t*)(S + gl.k[l]); ra.v = nullptr;
    ra.k_row = rpos;                                   // K,V land at the rows of their positions
    ra.d_model = d; ra.head_dim = hd; ra.kv_dim = kvd;
    ra.vt = (uint16_t*)(S + gl.vt[l]); ra.vt_ld = gl.vt_ld; ra.vt_col = rpos;
    ra.ssq_in = ssq_attn; ra.ssq_mul = ssq_mul; ra.eps = c->rms_eps; ra.ssq_clear = ssq_ffn;
    ra.skinny = 1; ra.w_stream = m->wqkv_s[l]; ra.w_blocked = 1;
    LZ_RUN(LAZYLLM_STEP_GEMM_QKV, l, M, 2.0 * M * (dd + 2.0 * kvd) * dd,
           launch_gemm(h, m->wqkv[l], nullptr, nullptr, M, d + 2 * kvd, d, d, d, 0, EPI_QKV_ROPE, st, &ra,
                       W + ws.gemm_ws, gemm_workspace_bytes()));
    LZ_RUN(LAZYLLM_STEP_ATTENTION, l, M, 4.0 * (double)M * (double)sel_count[s] * dd,
           launch_decode_attention(W + ws.q, rpos, M, S + gl.k[l], S + gl.vt[l], gl.vt_ld,
                                   s > 0 ? bits_of(s) : nullptr, n_tot, W + ws.o, H, hd, st,
                                   score_z(W + ws.score), score_zstat(W + ws.score, z_ld, H), z_ld,
                                   W + ws.att_ws, decode_attention_workspace_bytes(d, H), kv_group));
    EpiArgs eo{};
    eo.ssq_out = ssq_ffn; eo.skinny = 1; eo.w_stream = m->wo_s[l]; eo.w_blocked = 1;
    LZ_RUN(LAZYLLM_STEP_GEMM_O, l, M, 2.0 * M * dd * dd,
           launch_gemm(W + ws.o, m->wo[l], h, h, M, d, d, d, d, d, EPI_RESIDUAL, st, &eo,
                       W + ws.gemm_ws, gemm_workspace_bytes()));
    EpiArgs eg{};
    eg.ssq_in = ssq_ffn; eg.ssq_mul = ssq_mul; eg.eps = c->rms_eps; eg.ssq_clear = ssq_attn;
    eg.sf_z = score_z(W + ws.score);
    eg.sf_stat = (const float2*)score_zstat(W + ws.score, z_ld, H);
    eg.sf_s = scores_of(l);
    eg.sf_cu = nullptr; eg.sf_cu_z = nullptr;
    eg.sf_n_single = n_tot; eg.sf_heads = H; eg.sf_z_ld = z_ld;
    eg.sf_max_rows = n_tot; eg.sf_batch = 1;
    eg.skinny = 1; eg.w_stream = m->wgu_s[l]; eg.w_blocked = 1;
    LZ_RUN(LAZYLLM_STEP_GEMM_GATE_UP, l, M, 2.0 * M * 2.0 * (double)c->d_ffn * dd,
           launch_gemm(h, m->wgu[l], W + ws.act, nullptr, M, 2 * fp, d, d, d, fp, EPI_SWIGLU, st, &eg,
                       W + ws.gemm_ws, gemm_workspace_bytes()));
    EpiArgs ed{};
    ed.ssq_out = ssq_attn; ed.skinny = 1; ed.w_stream = m->wdown_s[l]; ed.w_blocked = 1;
    LZ_RUN(LAZYLLM_STEP_GEMM_DOWN, l, M, 2.0 * M * (double)c->d_ffn * dd,
           launch_gemm(W + ws.act, m->wdown[l], h, h, M, d, fp, fp, fp, d, EPI_RESIDUAL, st, &ed,
                       W + ws.gemm_ws, gemm_workspace_bytes()));
  }
  LZ_HIP(launch_gemm_exchange_check(W + ws.gemm_ws, res->status, st));
  if (lm_head_fused_fits(1, d)) {
    LZ_RUN(LAZYLLM_STEP_LM_HEAD, -1, 1, (double)c->vocab * rowb,
           launch_lm_head_fused(hbuf[cur], nullptr, M, 1, m->final_norm, m->lm_head, res->logits, d, c->vocab,
                                c->rms_eps, st));
  } else {
    LZ_RUN(LAZYLLM_STEP_LM_HEAD, -1, 1, (double)c->vocab * rowb,
           launch_final_norm(hbuf[cur], nullptr, M, 1, m->final_norm, (float*)(W + ws.xf), d,
                             c->rms_eps, st));
    LZ_RUN(LAZYLLM_STEP_LM_HEAD, -1, 1, 0.0,
           launch_lm_head((const float*)(W + ws.xf), m->lm_head, res->logits, 1, d, c->vocab, st));
  }
  g->n_tokens = n_tot;
  g->failed = false;
  return LAZYLLM_OK;
}

// ---- per-launch timing ---------------------------------------------------------------------

int lazyllm_profile_begin(void) {
  for (ProfRec& r : g_prof.recs) { g_prof.pool.push_back(r.start); g_prof.pool.push_back(r.stop); }
  g_prof.recs.clear();
  g_prof.on = true;
  return LAZYLLM_OK;
}

int lazyllm_profile_end(lazyllm_profile_record* out, int32_t capacity, int32_t* n_records) {
  g_prof.on = false;
  if (n_records == nullptr || capacity < 0 || (capacity > 0 && out == nullptr)) return LAZYLLM_EINVAL;
  int n = 0;
  for (ProfRec& r : g_prof.recs) {
    LZ_HIP(hipEventSynchronize(r.stop));
    float ms = 0.f;
    LZ_HIP(hipEventElapsedTime(&ms, r.start, r.stop));
    if (n < capacity) {
      out[n].step = r.step; out[n].layer = r.layer; out[n].rows = r.rows;
      out[n].ms = ms; out[n].work = r.work;
    }
    ++n;
  }
  *n_records = n;
  for (ProfRec& r : g_prof.recs) { g_prof.pool.push_back(r.start); g_prof.pool.push_back(r.stop); }
  g_prof.recs.clear();
  return LAZYLLM_OK;
}

// ---- single steps -------------------------------------------------------------------------

size_t lazyllm_op_gemm_workspace_bytes(void) { return gemm_workspace_bytes(); }

int lazyllm_op_gemm(const void* A, const void* W, void* C, const void* R, int32_t M, int32_t N,
                    int32_t K, int32_t lda, int32_t ldw, int32_t ldc, int32_t epilogue,
                    void* workspace, size_t ws_bytes, void* hip_stream) {
  if (!A || !W || !C || M < 0 || N <= 0 || K <= 0) return LAZYLLM_EINVAL;
  if (N % 128 != 0 || K % 64 != 0 || lda % 8 != 0 || ldw % 8 != 0 || ldc % 4 != 0)
    return LAZYLLM_EINVAL;
  if (lda < K || ldw < K) return LAZYLLM_EINVAL;
  const int epi = epilogue & 0xff;
  if (epilogue < 0 || epi > 2 || (epi == EPI_RESIDUAL && !R)) return LAZYLLM_EINVAL;
  if (ldc < (epi == EPI_SWIGLU ? N / 2 : N)) return LAZYLLM_EINVAL;
  if (M == 0) return LAZYLLM_OK;
  if (workspace != nullptr && ((uintptr_t)workspace & 255) != 0) return LAZYLLM_EINVAL;
  const int forced = (epilogue >> 8) & 0xff;
  if (forced == 8 && M > 32) return LAZYLLM_EINVAL;
  if ((forced == 8 || forced == 9 || forced == 10) && (workspace == nullptr || ws_bytes < gemm_workspace_bytes()))
    return LAZYLLM_EINVAL;
  EpiArgs ea{};
  if (workspace != nullptr && ws_bytes >= gemm_workspace_bytes()) {
    // the tickets of the weight-streaming kernel and the flags of the persistent stream-K kernel
    // live at the end of the workspace and must start at zero
    LZ_HIP(launch_gemm_counters_clear(workspace, (hipStream_t)hip_stream));
    ea.psk_ready = 1;
  }
  LZ_HIP(launch_gemm(A, W, C, R, M, N, K, lda, ldw, ldc, epilogue, (hipStream_t)hip_stream, &ea,
                     workspace, ws_bytes));
  return LAZYLLM_OK;
}

int lazyllm_op_gemm_rmsnorm(const void* A, const void* W, void* C, const void* R, int32_t M,
                            int32_t N, int32_t K, int32_t lda, int32_t ldw, int32_t ldc,
                            int32_t epilogue, const uint64_t* ssq_in, float eps, uint64_t* ssq_out,
                            uint64_t* ssq_clear, void* workspace, size_t ws_bytes,
                            void* hip_stream) {
  if (!A || !W || !C || M < 0 || N <= 0 || K <= 0) return LAZYLLM_EINVAL;
  if (N % 128 != 0 || K % 64 != 0 || lda % 8 != 0 || ldw % 8 != 0 || ldc % 4 != 0)
    return LAZYLLM_EINVAL;
  if (lda < K || ldw < K) return LAZYLLM_EINVAL;
  const int epi = epilogue & 0xff;
  if (epilogue < 0 || epi > 2 || (epi == EPI_RESIDUAL && !R)) return LAZYLLM_EINVAL;
  if (ldc < (epi == EPI_SWIGLU ? N / 2 : N)) return LAZYLLM_EINVAL;
  if ((ssq_in && (epi == EPI_RESIDUAL || !(eps > 0.f))) || (ssq_out && epi != EPI_RESIDUAL))
    return LAZYLLM_EINVAL;
  if (M == 0) return LAZYLLM_OK;
  if (workspace != nullptr && ((uintptr_t)workspace & 255) != 0) return LAZYLLM_EINVAL;
  EpiArgs ea{};
  ea.ssq_in = (const unsigned long long*)ssq_in;
  ea.ssq_mul = 1.0f / (4294967296.0f * (float)K);
  ea.eps = eps;
  ea.ssq_out = (unsigned long long*)ssq_out;
  ea.ssq_clear = (unsigned long long*)ssq_clear;
  // the 128x128 stream-K schedule has no row scaling or clearing: of the forms it may be chosen
  // for, only the plain residual one gets the workspace; the SiLU*mul form (tile walk, persistent
  // stream-K: both scale rows) always may
  const bool sk_ok = (!ssq_in && !ssq_clear) || epi == EPI_SWIGLU;
  const bool use_ws = sk_ok && workspace != nullptr && ws_bytes >= gemm_workspace_bytes();
  if (use_ws) {
    LZ_HIP(launch_gemm_counters_clear(workspace, (hipStream_t)hip_stream));
    ea.psk_ready = 1;
  }
  LZ_HIP(launch_gemm(A, W, C, R, M, N, K, lda, ldw, ldc, epilogue, (hipStream_t)hip_stream, &ea,
                     use_ws ? workspace : nullptr, use_ws ? ws_bytes : 0));
  return LAZYLLM_OK;
}

int lazyllm_op_pack_weight_stream(const void* W, int32_t N, int32_t K, int32_t ldw, void* packed,
                                  void* hip_stream) {
  if (!W || !packed || N <= 0 || K <= 0 || N % 128 != 0 || K % 64 != 0 || ldw % 8 != 0 || ldw < K ||
      ((uintptr_t)W & 15) != 0 || ((uintptr_t)packed & 15) != 0)
    return LAZYLLM_EINVAL;
  LZ_HIP(launch_pack_stream(W, N, K, ldw, packed, (hipStream_t)hip_stream));
  return LAZYLLM_OK;
}

int lazyllm_op_pack_weight_ksteps(const void* W, int32_t N, int32_t K, int32_t ldw, void* packed,
                                  void* hip_stream) {
  if (!W || !packed || N <= 0 || K <= 0 || K % 64 != 0 || ldw % 8 != 0 || ldw < K ||
      ((uintptr_t)W & 15) != 0 || ((uintptr_t)packed & 15) != 0)
    return LAZYLLM_EINVAL;
  LZ_HIP(launch_pack_kblock(W, N, K, ldw, packed, (hipStream_t)hip_stream));
  return LAZYLLM_OK;
}

int lazyllm_op_quantize_fp8(const void* x, int32_t rows, int32_t K, int32_t ldx, void* codes,
                            int32_t ldq, float* scale, void* hip_stream) {
  if (!x || !codes || !scale || rows < 0 || K <= 0 || K % 8 != 0 || K > 16384 || ldx < K || ldq < K ||
      ldx % 8 != 0 || ldq % 8 != 0 || ((uintptr_t)x & 15) != 0 || ((uintptr_t)codes & 7) != 0)
    return LAZYLLM_EINVAL;
  LZ_HIP(launch_quantize_rows_f8(x, rows, K, ldx, codes, ldq, scale, (hipStream_t)hip_stream));
  return LAZYLLM_OK;
}

int lazyllm_op_gemm_fp8(const void* a_codes, const float* a_scale, const void* w_codes,
                        const float* w_scale, void* C, const void* R, int32_t M, int32_t N, int32_t K,
                        int32_t lda, int32_t ldw, int32_t ldc, int32_t epilogue, void* hip_stream) {
  if (!a_codes || !a_scale || !w_codes || !w_scale || !C || M < 0 || N <= 0 || K <= 0)
    return LAZYLLM_EINVAL;
  if (N % 256 != 0 || K % 128 != 0 || lda % 16 != 0 || ldw % 16 != 0 || ldc % 4 != 0 || lda < K || ldw < K)
    return LAZYLLM_EINVAL;
  if (((uintptr_t)a_codes & 15) != 0 || ((uintptr_t)w_codes & 15) != 0 || ((uintptr_t)w_scale & 15) != 0)
    return LAZYLLM_EINVAL;
  if ((uint64_t)M * (uint64_t)lda >= (1ull << 32) || (uint64_t)N * (uint64_t)ldw >= (1ull << 32))
    return LAZYLLM_EINVAL;
  const bool blocked = (epilogue & (1 << 29)) != 0;   // w_codes K-step-major: [K / 128][N][128]
  if (epilogue >= 0) epilogue &= ~(1 << 29);
  if (epilogue < 0 || epilogue > 2 || (epilogue == EPI_RESIDUAL && !R)) return LAZYLLM_EINVAL;
  if (ldc < (epilogue == EPI_SWIGLU ? N / 2 : N)) return LAZYLLM_EINVAL;
  if (M == 0) return LAZYLLM_OK;
  EpiArgs ea{};
  ea.w_blocked = blocked ? 1 : 0;
  LZ_HIP(launch_gemm_f8(a_codes, a_scale, w_codes, w_scale, C, R, M, N, K, lda, ldw, ldc, epilogue,
                        (hipStream_t)hip_stream, &ea));
  return LAZYLLM_OK;
}

int lazyllm_op_rmsnorm(const void* h, const void* gain, void* x, int32_t rows, int32_t d, float eps,
                       void* hip_stream) {
  if (!h || !gain || !x || rows < 0 || d <= 0 || d % 8 != 0 || d > 16384 || !(eps > 0.f))
    return LAZYLLM_EINVAL;
  LZ_HIP(launch_rmsnorm(h, gain, x, rows, d, eps, (hipStream_t)hip_stream));
  return LAZYLLM_OK;
}

int lazyllm_op_qkv_rope(const void* x, const void* wqkv, const int32_t* pos, int32_t max_pos,
                        void* rope_table, void* q, void* k, void* v, int32_t rows, int32_t n_heads,
                        int32_t head_dim, float theta, void* hip_stream) {
  if (!x || !wqkv || !pos || !rope_table || !q || !k || !v || rows <= 0 || max_pos < 0 ||
      n_heads <= 0 || (head_dim != 64 && head_dim != 128) || (n_heads * head_dim) % 128 != 0 ||
      !(theta > 0.f))
    return LAZYLLM_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  const int d = n_heads * head_dim;
  LZ_HIP(launch_rope_table((float2*)rope_table, max_pos + 1, head_dim, theta, st));
  EpiArgs ra{};
  ra.pos = pos; ra.table = (const float2*)rope_table;
  ra.q = (uint16_t*)q; ra.k = (uint16_t*)k; ra.v = (uint16_t*)v;
  ra.d_model = d; ra.head_dim = head_dim;
  LZ_HIP(launch_gemm(x, wqkv, nullptr, nullptr, rows, 3 * d, d, d, d, 0, EPI_QKV_ROPE, st, &ra));
  return LAZYLLM_OK;
}

int lazyllm_op_v_transpose(const void* v, void* vt, int32_t vt_ld, int32_t rows, int32_t n_heads,
                           int32_t head_dim, void* hip_stream) {
  if (!v || !vt || rows <= 0 || n_heads <= 0 || (head_dim != 64 && head_dim != 128) ||
      vt_ld % 64 != 0 || vt_ld < (rows + 63) / 64 * 64)
    return LAZYLLM_EINVAL;
  LZ_HIP(launch_v_transpose(v, vt, nullptr, nullptr, rows, 1, rows, vt_ld, n_heads, head_dim,
                            (hipStream_t)hip_stream));
  return LAZYLLM_OK;
}

int lazyllm_op_attention(const void* q, const void* k, const void* vt, int32_t vt_ld, void* o,
                         int32_t rows, int32_t n_heads, int32_t head_dim, void* hip_stream) {
  if (!q || !k || !vt || !o || rows <= 0 || n_heads <= 0 || (head_dim != 64 && head_dim != 128) ||
      vt_ld % 64 != 0 || vt_ld < (rows + 63) / 64 * 64)
    return LAZYLLM_EINVAL;
  LZ_HIP(launch_attention(q, k, vt, o, nullptr, nullptr, rows, 1, rows, vt_ld, n_heads, head_dim,
                          (hipStream_t)hip_stream));
  return LAZYLLM_OK;
}

int lazyllm_op_attention_score(const void* q, const void* k, const void* vt, int32_t vt_ld, void* o,
                               float* s, void* scratch, int32_t rows, int32_t n_heads,
                               int32_t head_dim, void* hip_stream) {
  if (!q || !k || !vt || !o || !s || !scratch || rows <= 0 || n_heads <= 0 || n_heads > 256 ||
      (head_dim != 64 && head_dim != 128) || vt_ld % 64 != 0 || vt_ld < (rows + 63) / 64 * 64)
    return LAZYLLM_EINVAL;
  const int z_ld = (rows + 63) / 64 * 64;      // the scratch is sized for this padded length
  LZ_HIP(launch_attention(q, k, vt, o, nullptr, nullptr, rows, 1, rows, vt_ld, n_heads, head_dim,
                          (hipStream_t)hip_stream, score_z(scratch),
                          score_zstat(scratch, z_ld, n_heads), z_ld));
  LZ_HIP(launch_score_finish(s, scratch, nullptr, nullptr, rows, 1, z_ld, rows, n_heads,
                             (hipStream_t)hip_stream));
  return LAZYLLM_OK;
}

size_t lazyllm_op_score_scratch_bytes(int32_t rows, int32_t n_heads) {
  if (rows <= 0 || n_heads <= 0) return 0;
  return score_scratch_bytes(rows, 1, n_heads);
}

int lazyllm_op_score(const void* q_last, const void* k, float* s, void* scratch, int32_t rows,
                     int32_t n_heads, int32_t head_dim, void* hip_stream) {
  if (!q_last || !k || !s || !scratch || rows <= 0 || n_heads <= 0 || n_heads > 256 ||
      (head_dim != 64 && head_dim != 128) || (n_heads * head_dim) % 8 != 0 ||
      n_heads * head_dim > 8192)
    return LAZYLLM_EINVAL;
  // the kernel reads the query from row (rows-1) of a [rows, H*hd] tensor: rebase the pointer
  const char* qbase = (const char*)q_last - (size_t)(rows - 1) * n_heads * head_dim * 2;
  LZ_HIP(launch_score(qbase, k, s, scratch, nullptr, rows, 1, rows, rows, n_heads, head_dim,
                      (hipStream_t)hip_stream));
  return LAZYLLM_OK;
}

int lazyllm_op_select(const float* s, int32_t m, int32_t k, int32_t* keep_idx, int32_t* prune_idx,
                      void* hip_stream) {
  if (!s || !keep_idx || !prune_idx || m <= 0 || k < 1 || k > m) return LAZYLLM_EINVAL;
  LZ_HIP(launch_select(s, nullptr, nullptr, m, k, 1, keep_idx, prune_idx, (hipStream_t)hip_stream));
  return LAZYLLM_OK;
}

int lazyllm_op_gather(const void* h, const int32_t* pos, const int32_t* keep_idx, int32_t n_keep,
                      const int32_t* prune_idx, int32_t n_prune, void* h_out, int32_t* pos_out,
                      void* aux_h, int32_t* aux_pos, int32_t d, void* hip_stream) {
  if (!h || !pos || n_keep < 0 || n_prune < 0 || d <= 0 || d % 8 != 0) return LAZYLLM_EINVAL;
  if (n_keep > 0 && (!keep_idx || !h_out || !pos_out)) return LAZYLLM_EINVAL;
  if (n_prune > 0 && (!prune_idx || !aux_h || !aux_pos)) return LAZYLLM_EINVAL;
  LZ_HIP(launch_gather(h, pos, keep_idx, n_keep, prune_idx, n_prune, h_out, pos_out, aux_h, aux_pos,
                       d, (hipStream_t)hip_stream));
  return LAZYLLM_OK;
}

int lazyllm_op_lm_head(const void* h_last, const void* gain, const void* w_lm, float* xf,
                       float* logits, int32_t d, int32_t vocab, float eps, void* hip_stream) {
  if (!h_last || !gain || !w_lm || !xf || !logits || d <= 0 || d % 8 != 0 || vocab <= 0 ||
      !(eps > 0.f))
    return LAZYLLM_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  if (lm_head_fused_fits(1, d)) {
    // (one launch: every workgroup normalises the row itself; xf is then not used)
    LZ_HIP(launch_lm_head_fused(h_last, nullptr, 1, 1, gain, w_lm, logits, d, vocab, eps, st));
    return LAZYLLM_OK;
  }
  LZ_HIP(launch_final_norm(h_last, nullptr, 1, 1, gain, xf, d, eps, st));
  LZ_HIP(launch_lm_head(xf, w_lm, logits, 1, d, vocab, st));
  return LAZYLLM_OK;
}

}  // extern "C"
