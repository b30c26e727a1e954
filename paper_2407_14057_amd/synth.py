"""Seeded synthetic inputs: model shapes, weights, prompts, keep schedules.

This module only draws random numbers and lays them out; it holds none of the
method's arithmetic.  The same buffers it returns are handed to the HIP path
and to the CPU checker, so both see identical bytes.

Workload recipe (stands in for LongBench prompts, whose mean length is the
3376 tokens quoted in the paper's introduction):
  * weights  : every projection / embedding / LM-head matrix ~ N(0, 0.02),
               stored as bf16 (round-to-nearest-even of an fp32 draw);
               RMSNorm gains are 1.0
  * prompts  : token ids uniform over the vocabulary
  * needles  : optional per-position embedding scale (x8 at 64 positions)
  * schedules: (layer, keep_permille) pairs; permille is of the tokens that
               survive so far
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

import numpy as np
import torch


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    n_kv_heads: int = 0            # K,V heads; 0 = as many as query heads (no grouped-query attention)
    gemm_dtype: int = 0            # projections of the prefill: 0 = 16-bit floats, 1 = the 8-bit (OFP8 E4M3) variant

    @property
    def kv_heads(self) -> int:
        return self.n_kv_heads if self.n_kv_heads else self.n_heads

    def as_dict(self) -> Dict[str, float]:
        return dict(n_layers=self.n_layers, d_model=self.d_model, n_heads=self.n_heads,
                    head_dim=self.head_dim, d_ffn=self.d_ffn, vocab=self.vocab,
                    rms_eps=self.rms_eps, rope_theta=self.rope_theta, n_kv_heads=self.kv_heads,
                    gemm_dtype=self.gemm_dtype)


TINY = ModelShape(n_layers=4, d_model=256, n_heads=4, head_dim=64, d_ffn=688, vocab=1024)
LLAMA7B = ModelShape(n_layers=32, d_model=4096, n_heads=32, head_dim=128, d_ffn=11008, vocab=32000)
# the paper's second model: the same decoder stack with a 51200-entry vocabulary and eps 1e-6
# a grouped-query variant at 8B scale (Llama-3-8B-like: 8 K,V heads for 32 query heads, wider MLP and vocabulary)
GQA8B = ModelShape(n_layers=32, d_model=4096, n_heads=32, head_dim=128, d_ffn=14336, vocab=128256,
                   rope_theta=500000.0, n_kv_heads=8)
XGEN7B = ModelShape(n_layers=32, d_model=4096, n_heads=32, head_dim=128, d_ffn=11008, vocab=51200, rms_eps=1e-6)
# the same models with the projections in the 8-bit variant
TINY_FP8 = ModelShape(n_layers=4, d_model=256, n_heads=4, head_dim=64, d_ffn=688, vocab=1024, gemm_dtype=1)
LLAMA7B_FP8 = ModelShape(n_layers=32, d_model=4096, n_heads=32, head_dim=128, d_ffn=11008, vocab=32000, gemm_dtype=1)


@dataclass(frozen=True)
class Workload:
    name: str
    shape: ModelShape
    weight_seed: int
    prompt_seed: int
    seqlens: Tuple[int, ...]
    schedule: Tuple[Tuple[int, int], ...]          # (layer, keep_permille of survivors)
    needle_seed: int = 0
    n_needles: int = 0
    needle_scale: float = 8.0


def _batch_lengths(seed: int, batch: int, lo: int, hi: int) -> Tuple[int, ...]:
    rng = np.random.Generator(np.random.PCG64(seed))
    return tuple(int(x) for x in rng.integers(lo, hi + 1, size=batch))


WORKLOADS: Dict[str, Workload] = {
    # small case the CPU checker finishes in seconds
    "tiny512": Workload("tiny512", TINY, 1001, 2001, (512,), ((2, 700), (3, 500))),
    # headline: 7B shape, 3376-token prompt
    "7b_3376": Workload("7b_3376", LLAMA7B, 1002, 2002, (3376,), ((8, 700), (16, 500), (24, 300))),
    "7b_8192": Workload("7b_8192", LLAMA7B, 1002, 2003, (8192,), ((8, 600), (16, 400), (24, 200))),
    "7b_3376_needles": Workload("7b_3376_needles", LLAMA7B, 1002, 2004, (3376,),
                                ((4, 500), (12, 500), (20, 500)), needle_seed=3004, n_needles=64),
    "xgen7b_3376": Workload("xgen7b_3376", XGEN7B, 1003, 2006, (3376,), ((8, 700), (16, 500), (24, 300))),
    "gqa8b_3376": Workload("gqa8b_3376", GQA8B, 1004, 2007, (3376,), ((8, 700), (16, 500), (24, 300))),
    "7b_batch8": Workload("7b_batch8", LLAMA7B, 1002, 2005, _batch_lengths(4005, 8, 1024, 8192),
                          ((8, 700), (16, 500), (24, 300))),
    # the small and the headline case with the projections in the 8-bit variant (same weights, same prompts)
    "tiny512_fp8": Workload("tiny512_fp8", TINY_FP8, 1001, 2001, (512,), ((2, 700), (3, 500))),
    "7b_3376_fp8": Workload("7b_3376_fp8", LLAMA7B_FP8, 1002, 2002, (3376,), ((8, 700), (16, 500), (24, 300))),
}

_PER_LAYER = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


def weight_shapes(s: ModelShape) -> Dict[str, Tuple[int, ...]]:
    """Shape of each tensor, nn.Linear convention [out_features, in_features]."""
    d, f = s.d_model, s.d_ffn
    kvd = s.kv_heads * s.head_dim
    return {
        "embed": (s.vocab, d), "final_norm": (d,), "lm_head": (s.vocab, d),
        "attn_norm": (d,), "ffn_norm": (d,),
        "wq": (d, d), "wk": (kvd, d), "wv": (kvd, d), "wo": (d, d),
        "w_gate": (f, d), "w_up": (f, d), "w_down": (d, f),
    }


def make_weights(s: ModelShape, seed: int, device: str = "cpu", std: float = 0.02,
                 gain_jitter: float = 0.0) -> Dict[str, object]:
    """bf16 tensors: {'embed','final_norm','lm_head'} and per-layer lists.

    Draws are fp32 N(0, std) from a torch generator on `device`, rounded once to
    bf16.  The CPU and GPU generators give different streams, so a workload must
    always be generated on one device and copied (the headline 7B weights are
    drawn on the GPU, the tiny ones on the CPU).  gain_jitter > 0 makes the norm
    gains 1 + U(-j, j) instead of exactly 1 (used by tests that must notice a
    missing gain).
    """
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    shapes = weight_shapes(s)

    def draw(name: str) -> torch.Tensor:
        shp = shapes[name]
        if name.endswith("norm"):
            if gain_jitter > 0.0:
                u = torch.rand(shp, generator=gen, device=device, dtype=torch.float32)
                return (1.0 + gain_jitter * (2.0 * u - 1.0)).to(torch.bfloat16)
            return torch.ones(shp, device=device, dtype=torch.bfloat16)
        w = torch.empty(shp, device=device, dtype=torch.float32)
        w.normal_(0.0, std, generator=gen)
        return w.to(torch.bfloat16)

    out: Dict[str, object] = {"embed": draw("embed")}
    for name in _PER_LAYER:
        out[name] = []
    for _ in range(s.n_layers):
        for name in _PER_LAYER:
            out[name].append(draw(name))
    out["final_norm"] = draw("final_norm")
    out["lm_head"] = draw("lm_head")
    return out


def weights_to_host_bits(w: Dict[str, object]) -> Dict[str, object]:
    """Same weights as numpy uint16 arrays holding the bf16 bit patterns."""
    def bits(t: torch.Tensor) -> np.ndarray:
        return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
    out: Dict[str, object] = {}
    for k, v in w.items():
        out[k] = [bits(t) for t in v] if isinstance(v, list) else bits(v)
    return out


def layer_to_host_bits(w: Dict[str, object], layer: int) -> Dict[str, np.ndarray]:
    """One layer's tensors as bf16 bit patterns (avoids copying all 13 GB)."""
    def bits(t: torch.Tensor) -> np.ndarray:
        return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
    return {name: bits(w[name][layer]) for name in _PER_LAYER}


def make_prompt(n: int, vocab: int, seed: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(0, vocab, size=n, dtype=np.int64).astype(np.int32)


def make_needle_scale(n: int, n_needles: int, seed: int, scale: float = 8.0) -> np.ndarray:
    """fp32[n], 1.0 everywhere except `n_needles` distinct random positions."""
    rng = np.random.Generator(np.random.PCG64(seed))
    pos = rng.choice(n, size=n_needles, replace=False)
    out = np.ones(n, dtype=np.float32)
    out[pos] = scale
    return out


def make_workload_inputs(wl: Workload) -> Dict[str, object]:
    """Token ids (packed over the batch), cu_seqlens and optional embed scale."""
    ids: List[np.ndarray] = []
    scales: List[np.ndarray] = []
    for b, n in enumerate(wl.seqlens):
        ids.append(make_prompt(n, wl.shape.vocab, wl.prompt_seed + b))
        if wl.n_needles:
            scales.append(make_needle_scale(n, wl.n_needles, wl.needle_seed + b, wl.needle_scale))
    cu = np.zeros(len(wl.seqlens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(np.asarray(wl.seqlens, dtype=np.int64))
    return {
        "token_ids": np.concatenate(ids).astype(np.int32),
        "cu_seqlens": cu,
        "embed_scale": np.concatenate(scales).astype(np.float32) if scales else None,
    }


# --- score vectors for the selection kernel -------------------------------------------------

def make_scores(kind: str, n: int, seed: int) -> np.ndarray:
    """Non-negative fp32 score vectors with the shapes selection must survive."""
    rng = np.random.Generator(np.random.PCG64(seed))
    if kind == "uniform":
        s = rng.random(n)
    elif kind == "softmax_like":           # mean-of-softmax rows: positive, sums to 1
        z = rng.normal(0.0, 1.6, size=(8, n))
        e = np.exp(z - z.max(axis=1, keepdims=True))
        s = (e / e.sum(axis=1, keepdims=True)).mean(axis=0)
    elif kind == "lognormal3":
        s = rng.lognormal(0.0, 3.0, size=n)
        s = s / s.sum()
    elif kind == "pareto":
        s = rng.pareto(1.1, size=n)
        s = s / s.sum()
    elif kind == "spikes":                 # 64 spikes at 1000x the median
        s = rng.random(n) * 0.1 + 1.0
        idx = rng.choice(n, size=min(64, n), replace=False)
        s[idx] *= 1000.0
        s = s / s.sum()
    elif kind == "few_values":             # many exact duplicates
        s = rng.choice(np.asarray([0.0, 1e-6, 0.25, 0.5, 1.0]), size=n)
    elif kind == "all_equal":
        s = np.full(n, 1.0 / max(n, 1))
    elif kind == "denormal_zero":          # zeros and denormals from exp underflow
        s = rng.random(n)
        s[rng.random(n) < 0.3] = 0.0
        m = rng.random(n) < 0.3
        s[m] = s[m] * 1e-41
    else:
        raise ValueError(kind)
    return np.ascontiguousarray(s, dtype=np.float32)


SCORE_KINDS = ("uniform", "softmax_like", "lognormal3", "pareto", "spikes", "few_values",
               "all_equal", "denormal_zero")
