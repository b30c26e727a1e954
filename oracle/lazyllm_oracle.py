"""CPU checker for LazyLLM's pruned prefill -- TEST INFRASTRUCTURE ONLY.

A plain, slow numpy implementation of what the prefill stage with progressive
token pruning computes (paper Sec. 3.1 "Background on LLM Inference", Sec. 3.2
"Inference with LazyLLM": Eq. 1, the top-k percentile rule, the Aux Cache).
It exists so the HIP path can be compared against something written straight
from the paper.  Only tests, the smoke check and the benchmark's cpu_baseline
leg may import it; it shares no code with the HIP path and imports nothing
from it.

Arithmetic is fp64 by default (dtype=np.float32 gives the fp32 variant).  The
weights arrive as bf16 bit patterns (uint16) or as float arrays; bf16 bits are
widened exactly.

The paper prints no pseudo-code and no worked numbers.  Readings taken where it
is silent (each also listed in the design notes):
  * Eq. 1's A[h, i, N] is the probability that the LAST token (query N)
    attends to token i, i.e. the last row of the usual [query, key] map.
  * "pruned at layer l+1 by the scores of layer l": scores of layer p-1 decide
    which tokens ENTER layer p.  Keep ratios are fractions of the tokens that
    still survive, and the kept count is ceil(ratio * m), in integer
    arithmetic on permille, never below 1.
  * the last token is always kept and counts towards k; ties are broken
    towards the lower index; the comparison is done on fp32 scores.
  * softmax for Eq. 1 runs over the tokens present at that layer.
  * kept tokens keep their ORIGINAL position ids for RoPE (half-split pairing,
    theta^(-2i/hd)).
  * the Aux Cache of pruning layer p holds the layer-p INPUT hidden state and
    the original position of every token dropped there.
  * model fine print (only "Llama 2, 32 layers, width 4096" is stated):
    pre-norm RMSNorm, multi-head attention, SwiGLU MLP, untied LM head, no bias.
    Grouped-query attention (fewer K,V heads than query heads, each shared by a
    group) is accepted as a model variant: Eq. 1 stays the mean over all query
    heads' maps.

Parity pins for each function live in tests/test_oracle_*.py (library
transformer, closed forms, brute force, invariants).  Absolute logits of the
random 7B-shaped model have no external reference: they are pinned only
transitively through the same code passing those tests at the small shape.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np


# ------------------------------------------------------------------ number formats

def bf16_bits_to_float(bits: np.ndarray, dtype=np.float64) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) exactly."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(dtype)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bf16 value (ties to even), result in x's dtype.

    Models a store of an fp32 register to a bf16 tensor.
    """
    x = np.asarray(x)
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    r = ((u + bias) & np.uint32(0xFFFF0000)).view(np.float32)
    return r.astype(x.dtype).reshape(x.shape)


def _as_float(w, dtype) -> np.ndarray:
    w = np.asarray(w)
    if w.dtype == np.uint16:
        return bf16_bits_to_float(w, dtype)
    return w.astype(dtype)


# ------------------------------------------------------------------ transformer pieces

def rmsnorm(h: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """x = h / sqrt(mean(h^2) + eps) * gain, per row (Llama's RMSNorm)."""
    ms = np.mean(h * h, axis=-1, keepdims=True)
    return h / np.sqrt(ms + eps) * gain


def rope(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding on x[m, H, hd] at integer positions pos[m].

    Dimension i pairs with i + hd/2; the pair is rotated by pos * theta^(-2i/hd).
    Angles are always formed in fp64.
    """
    m, H, hd = x.shape
    half = hd // 2
    inv_freq = np.float64(theta) ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = pos.astype(np.float64)[:, None] * inv_freq[None, :]          # [m, half]
    c = np.cos(ang).astype(x.dtype)[:, None, :]
    s = np.sin(ang).astype(x.dtype)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def softmax_rows(z: np.ndarray) -> np.ndarray:
    """Row softmax with the row maximum subtracted first."""
    z = z - np.max(z, axis=-1, keepdims=True)
    e = np.exp(z)
    return e / np.sum(e, axis=-1, keepdims=True)


def attention_map(q: np.ndarray, k: np.ndarray) -> np.ndarray:
    """One head's causal attention probabilities P[query, key], q,k: [m, hd].

    Row j is token j's distribution over tokens 0..j (Sec. 3.1: causal
    self-attention; Eq. 1's A^l for one head, indexed [query, key]).
    """
    m, hd = q.shape
    z = (q @ k.T) / math.sqrt(hd)
    z = np.where(np.tril(np.ones((m, m), dtype=bool)), z, -np.inf)
    return softmax_rows(z)


def causal_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Multi-head causal attention and Eq. 1 scores.

    q: [m, H, hd]; k, v: [m, Hkv, hd] with Hkv dividing H (grouped-query attention: query head h
    reads K,V head h // (H / Hkv); Hkv = H is plain multi-head attention).  Returns
    (o[m, H, hd], s[m]) where s_i = (1/H) sum_h A_h[last query, key i]   (Eq. 1, the mean over
    all H attention maps).  The full m x m map of each head is materialised, as in the definition.
    """
    m, H, hd = q.shape
    group = H // k.shape[1]
    o = np.empty_like(q)
    s = np.zeros(m, dtype=q.dtype)
    for head in range(H):
        P = attention_map(q[:, head, :], k[:, head // group, :])
        o[:, head, :] = P @ v[:, head // group, :]
        s += P[m - 1, :]
    return o, s / H


def last_row_scores(q_last: np.ndarray, k: np.ndarray) -> np.ndarray:
    """Eq. 1 from the last query alone: q_last[H, hd], k[m, Hkv, hd] -> s[m].

    The last row of a causal map has no masked entry, so it is the plain
    softmax of q_last . k_i / sqrt(hd) over all m tokens, then the head mean.
    """
    m, Hkv, hd = k.shape
    kk = np.repeat(k, q_last.shape[0] // Hkv, axis=1)
    z = np.einsum("hd,mhd->hm", q_last, kk) / math.sqrt(hd)
    return np.mean(softmax_rows(z), axis=0)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def swiglu(y: np.ndarray, w_gate: np.ndarray, w_up: np.ndarray) -> np.ndarray:
    """silu(y Wg^T) * (y Wu^T)."""
    return silu(y @ w_gate.T) * (y @ w_up.T)


# ------------------------------------------------------------------ pruning pieces

def keep_count(m: int, permille: int) -> int:
    """Tokens kept out of m at a keep ratio of permille/1000: ceil, at least 1."""
    if not (0 < permille <= 1000):
        raise ValueError("keep_permille must be in (0, 1000]")
    return max(1, (m * permille + 999) // 1000)


def keep_counts(n: int, n_layers: int, schedule: Sequence[Tuple[int, int]]) -> List[int]:
    """Tokens that run each layer, for a prompt of n tokens (progressive pruning)."""
    sched = dict(schedule)
    out, m = [], n
    for l in range(n_layers):
        if l in sched:
            m = keep_count(m, sched[l])
        out.append(m)
    return out


def select_tokens(scores: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """Top-k percentile rule on the scores of the m tokens of the previous layer.

    Keeps the last token plus the k-1 best of the others; "best" is higher
    fp32 score, then lower index.  Returns (kept, pruned) local indices, both
    ascending.
    """
    s = np.asarray(scores).astype(np.float32)
    m = s.shape[0]
    if not (1 <= k <= m):
        raise ValueError("k out of range")
    order = np.argsort(-s[: m - 1], kind="stable")        # descending score, ascending index
    kept = np.sort(np.concatenate([order[: k - 1], np.asarray([m - 1], dtype=order.dtype)]))
    mask = np.ones(m, dtype=bool)
    mask[kept] = False
    return kept.astype(np.int64), np.nonzero(mask)[0].astype(np.int64)


# ------------------------------------------------------------------ the layer and the prefill

class LayerWeights:
    """One decoder layer's matrices widened to the working dtype."""

    def __init__(self, weights: Dict[str, object], l: int, dtype):
        for name in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down"):
            setattr(self, name, _as_float(weights[name][l], dtype))


def projection_8bit(a: np.ndarray, w: np.ndarray, gain: Optional[np.ndarray] = None,
                    eps: float = 0.0) -> np.ndarray:
    """A projection as the 8-bit GEMM variant defines it (an extension; the paper's models
    compute in 16-bit floating point): rows of `a` and rows of the stored weight are quantised
    to OFP8 E4M3 with one scale per row (fp8_oracle.quantize_rows) and multiplied
    (fp8_oracle.gemm_fp8).  With `gain`, the projection is that of RMSNorm(a): the gain is folded
    into the stored 16-bit weight, w' = bf16(w * gain), the UNnormalised rows of `a` are what
    is quantised, and 1/rms(a) scales the product's rows."""
    from . import fp8_oracle as F8
    wf = w if gain is None else round_to_bf16(w * gain[None, :])
    ac, sa = F8.quantize_rows(a)
    wc, sw = F8.quantize_rows(wf)
    y = F8.gemm_fp8(ac, sa, wc, sw)
    if gain is not None:
        y = y / np.sqrt(np.mean(a * a, axis=-1, keepdims=True) + eps)
    return y


def decoder_layer(h: np.ndarray, pos: np.ndarray, lw: LayerWeights, n_heads: int, head_dim: int,
                  eps: float, theta: float, store=lambda t: t, gemm8: bool = False):
    """One pre-norm Llama layer on m tokens with original positions pos.

    `store` is applied wherever a tensor is written back to memory (identity,
    or round_to_bf16 to model bf16 activations).  Returns (h_out, k, v, s) with
    k, v [m, Hkv, hd] as they enter the KV cache (Hkv = rows of wk / hd) and s the Eq. 1 scores.
    gemm8: the four projections run as projection_8bit (everything else is unchanged).
    """
    m, d = h.shape
    n_kv_heads = lw.wk.shape[0] // head_dim          # grouped-query attention when below n_heads
    kvd = n_kv_heads * head_dim
    # The normalised activations x and y are not rounding points: the data flow being modelled
    # folds RMSNorm into the projections and never writes them to memory.
    if gemm8:
        qkv = projection_8bit(h, np.concatenate([lw.wq, lw.wk, lw.wv], axis=0), lw.attn_norm, eps)
        q = qkv[:, :d].reshape(m, n_heads, head_dim)
        k = qkv[:, d:d + kvd].reshape(m, n_kv_heads, head_dim)
        v = store(qkv[:, d + kvd:].reshape(m, n_kv_heads, head_dim))
    else:
        x = rmsnorm(h, lw.attn_norm, eps)
        q = (x @ lw.wq.T).reshape(m, n_heads, head_dim)
        k = (x @ lw.wk.T).reshape(m, n_kv_heads, head_dim)
        v = store((x @ lw.wv.T).reshape(m, n_kv_heads, head_dim))
    q = store(rope(q, pos, theta))
    k = store(rope(k, pos, theta))
    o, s = causal_attention(q, k, v)
    o = store(o)
    if gemm8:
        h = store(h + projection_8bit(o.reshape(m, d), lw.wo))
        f = lw.w_gate.shape[0]
        gu = projection_8bit(h, np.concatenate([lw.w_gate, lw.w_up], axis=0), lw.ffn_norm, eps)
        a = store(silu(gu[:, :f]) * gu[:, f:])
        h = store(h + projection_8bit(a, lw.w_down))
        return h, k, v, s
    h = store(h + o.reshape(m, d) @ lw.wo.T)
    y = rmsnorm(h, lw.ffn_norm, eps)
    a = store(swiglu(y, lw.w_gate, lw.w_up))
    h = store(h + a @ lw.w_down.T)
    return h, k, v, s


class PrefillResult:
    def __init__(self):
        self.logits: Optional[np.ndarray] = None          # [V]
        self.kept_pos: List[np.ndarray] = []               # per layer, original positions, ascending
        self.k: List[np.ndarray] = []                      # per layer [n_l, H, hd]
        self.v: List[np.ndarray] = []
        self.scores: List[np.ndarray] = []                 # per layer [n_l]  (Eq. 1)
        self.aux_pos: Dict[int, np.ndarray] = {}           # pruning layer -> positions dropped there
        self.aux_h: Dict[int, np.ndarray] = {}             # pruning layer -> their hidden states
        self.hidden_in: List[np.ndarray] = []              # per layer input h (only if keep_hidden)
        self.hidden_out: Optional[np.ndarray] = None       # last layer output


def prefill(shape: Dict[str, float], weights: Dict[str, object], token_ids: np.ndarray,
            schedule: Sequence[Tuple[int, int]], *, dtype=np.float64, bf16_storage: bool = False,
            forced_keep: Optional[Dict[int, np.ndarray]] = None,
            embed_scale: Optional[np.ndarray] = None, n_layers: Optional[int] = None,
            keep_hidden: bool = False, gemm8: bool = False) -> PrefillResult:
    """Prefill one prompt with progressive token pruning.

    shape: dict with n_layers, d_model, n_heads, head_dim, d_ffn, vocab, rms_eps,
    rope_theta.  schedule: (layer, keep_permille) pairs, layer >= 1.
    forced_keep: {layer: original positions to keep there} overrides the
    oracle's own choice at that layer (for comparing downstream of a near-tie).
    n_layers: run only the first n_layers layers (bounded timing samples).
    gemm8: the layers' projections in the 8-bit variant (see projection_8bit).
    """
    L = int(shape["n_layers"]) if n_layers is None else int(n_layers)
    H, hd = int(shape["n_heads"]), int(shape["head_dim"])
    eps, theta = float(shape["rms_eps"]), float(shape["rope_theta"])
    store = round_to_bf16 if bf16_storage else (lambda t: t)
    sched = dict(schedule)
    for l in sched:
        if not (1 <= l < int(shape["n_layers"])):
            raise ValueError("pruning layer must be in [1, L-1]: layer 0 has no prior scores")

    ids = np.asarray(token_ids, dtype=np.int64)
    N = ids.shape[0]
    h = _as_float(np.asarray(weights["embed"])[ids], dtype)
    if embed_scale is not None:
        h = store(h * np.asarray(embed_scale, dtype=dtype)[:, None])
    pos = np.arange(N, dtype=np.int64)
    res = PrefillResult()
    s_prev = None
    for l in range(L):
        if l in sched and sched[l] < 1000:
            m = h.shape[0]
            k_keep = keep_count(m, sched[l])
            if forced_keep is not None and l in forced_keep:
                want = np.asarray(forced_keep[l], dtype=np.int64)
                kept = np.searchsorted(pos, want)
                if (kept.shape[0] != k_keep or np.any(kept >= m) or np.any(pos[kept] != want)
                        or np.any(np.diff(want) <= 0) or want[-1] != pos[-1]):
                    raise ValueError("forced kept set is not a valid selection at layer %d" % l)
                mask = np.ones(m, dtype=bool)
                mask[kept] = False
                pruned = np.nonzero(mask)[0]
            else:
                kept, pruned = select_tokens(s_prev, k_keep)
            res.aux_pos[l] = pos[pruned].copy()
            res.aux_h[l] = h[pruned].copy()
            h, pos = h[kept], pos[kept]
        if keep_hidden:
            res.hidden_in.append(h.copy())
        lw = LayerWeights(weights, l, dtype)
        h, k, v, s_prev = decoder_layer(h, pos, lw, H, hd, eps, theta, store, gemm8)
        res.kept_pos.append(pos.copy())
        res.k.append(k)
        res.v.append(v)
        res.scores.append(s_prev)
    res.hidden_out = h
    xf = rmsnorm(h[-1], _as_float(weights["final_norm"], dtype), eps)
    res.logits = _as_float(weights["lm_head"], dtype) @ xf
    return res


def prefill_batch(shape, weights, token_ids: np.ndarray, cu_seqlens: np.ndarray, schedule,
                  **kw) -> List[PrefillResult]:
    """Independent prompts packed back to back; each is pruned on its own."""
    out = []
    scale = kw.pop("embed_scale", None)
    forced = kw.pop("forced_keep", None)
    for b in range(len(cu_seqlens) - 1):
        lo, hi = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        out.append(prefill(shape, weights, token_ids[lo:hi], schedule,
                           embed_scale=None if scale is None else scale[lo:hi],
                           forced_keep=None if forced is None else forced[b], **kw))
    return out


def decision_margin(scores: np.ndarray, k: int, rel: float = 1e-3):
    """Which candidates are safely above / below the selection threshold.

    tau = the (k-1)-th largest score among tokens 0..m-2 (the last token is
    forced).  Token j is 'decided' when |s_j - tau| > rel * tau.  Returns
    (tau, decided_mask[m]); the last token is always decided.
    """
    s = np.asarray(scores, dtype=np.float64)
    m = s.shape[0]
    decided = np.ones(m, dtype=bool)
    if k - 1 <= 0 or k >= m:
        return (math.inf if k - 1 <= 0 else 0.0), decided
    cand = np.sort(s[: m - 1])[::-1]
    tau = cand[k - 2]
    decided[: m - 1] = np.abs(s[: m - 1] - tau) > rel * tau
    return tau, decided
