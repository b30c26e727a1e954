"""CPU checker for LazyLLM's decoding steps with the Aux Cache -- TEST INFRASTRUCTURE ONLY.

A plain, slow numpy implementation of one generation step after a pruned
prefill (paper Sec. 3.2 "Inference with LazyLLM": progressive pruning applied in
every generation step, Eq. 1, and the paragraph "Aux Cache").  Only tests, the
smoke check and the benchmark's cpu_baseline leg may import it; it shares no
code with the HIP path.  It builds on the prefill checker in this package.

The paper describes the decoding steps in prose and one figure, with no
pseudo-code.  What this module computes, step by step, and the readings taken
where the text is silent:

  * A step feeds ONE new token (chosen by the caller from the previous logits)
    at the next original position.  It is the step's last token: its attention
    row defines Eq. 1's scores, and it is never pruned.
  * Every step selects afresh.  Candidates at layer 0 are all tokens so far.  At
    a pruning layer p the same top-k percentile rule as in the prefill is
    applied to the candidates of layer p-1, with this step's scores of layer
    p-1 (k = ceil(ratio * candidates), last token forced, ties to the lower
    position).  A token pruned in an earlier step may be selected again.
  * A selected token whose K,V exist at the layer is read from the KV cache.  One
    whose K,V do not exist is REVIVED: its layer input is the hidden state it
    carried out of the previous layer in this same step, or else the Aux Cache
    entry of this layer (the state it had when it was pruned here).  Revived
    tokens run the layer exactly like the new token (RMSNorm, projections, RoPE
    at the original position, attention, MLP), and their K,V stay in the cache,
    so no token is computed twice in any layer.
  * Attention of every token that runs the layer is causal over the tokens
    SELECTED at that layer in this step (those at or before its own position).
  * A token that ran layer p-1 in this step, is not selected at pruning layer p
    and has no K,V there leaves its hidden state in the Aux Cache of layer p.
  * Generated tokens are ordinary tokens in later steps.

Pins live in tests/test_oracle_decode.py: without pruning a step must reproduce
the prefill checker on the prompt extended by one token; reviving every token
at the first pruning layer must reproduce the dense K,V and scores of that
layer; single-row steps are checked against a hand-written softmax; and the
"at most once per layer" / nesting / counting invariants are checked over
several steps.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import lazyllm_oracle as P


class StepResult:
    def __init__(self):
        self.logits: Optional[np.ndarray] = None      # [V], distribution of the token after the new one
        self.selected: List[np.ndarray] = []          # per layer: positions selected in this step, ascending
        self.ran: List[np.ndarray] = []               # per layer: positions that ran the layer (new token last)
        self.scores: List[np.ndarray] = []            # per layer: Eq. 1 over `selected`
        self.hidden_out: Optional[np.ndarray] = None  # last layer's output rows, ordered like ran[-1]


class Generation:
    """KV cache and Aux Cache of one sequence, indexed by original position."""

    def __init__(self, shape: Dict[str, float], weights: Dict[str, object], schedule: Sequence[Tuple[int, int]],
                 prefill_result: P.PrefillResult, n_prompt: int, capacity: int, *, dtype=np.float64,
                 bf16_storage: bool = False):
        self.shape, self.weights, self.dtype = shape, weights, dtype
        self.L = int(shape["n_layers"])
        self.H, self.hd, self.d = int(shape["n_heads"]), int(shape["head_dim"]), int(shape["d_model"])
        self.eps, self.theta = float(shape["rms_eps"]), float(shape["rope_theta"])
        self.store = P.round_to_bf16 if bf16_storage else (lambda t: t)
        self.schedule = [(int(l), int(r)) for l, r in schedule]
        self.n_prompt, self.n_tokens, self.cap = int(n_prompt), int(n_prompt), int(capacity)
        if capacity < n_prompt:
            raise ValueError("capacity below the prompt length")
        self.Hkv = int(np.asarray(weights["wk"][0]).shape[0]) // self.hd     # K,V heads (grouped-query models)
        self.k = [np.full((capacity, self.Hkv, self.hd), np.nan, dtype=dtype) for _ in range(self.L)]
        self.v = [np.full((capacity, self.Hkv, self.hd), np.nan, dtype=dtype) for _ in range(self.L)]
        self.has_kv = [np.zeros(capacity, dtype=bool) for _ in range(self.L)]
        self.aux_h = [np.full((capacity, self.d), np.nan, dtype=dtype) for _ in range(self.L)]
        self.has_aux = [np.zeros(capacity, dtype=bool) for _ in range(self.L)]
        self.times_computed = np.zeros((self.L, capacity), dtype=np.int64)
        for l in range(self.L):
            pos = np.asarray(prefill_result.kept_pos[l], dtype=np.int64)
            self.k[l][pos], self.v[l][pos] = prefill_result.k[l], prefill_result.v[l]
            self.has_kv[l][pos] = True
            self.times_computed[l, pos] += 1
        for l, pos in prefill_result.aux_pos.items():
            self.aux_h[l][pos] = prefill_result.aux_h[l]
            self.has_aux[l][pos] = True

    def prompt_tokens_computed(self) -> float:
        """Share of (prompt token, layer) pairs whose K,V have been computed so far."""
        return float(np.mean([hk[: self.n_prompt].mean() for hk in self.has_kv]))

    def step(self, token_id: int, *, schedule: Optional[Sequence[Tuple[int, int]]] = None,
             forced_selected: Optional[Dict[int, np.ndarray]] = None) -> StepResult:
        """One generation step on `token_id`.

        schedule: keep schedule of this step (default: the one given at construction).
        forced_selected: {pruning layer: positions} replaces the top-k choice there
        (for comparing downstream of a near-tie); it must be a valid selection.
        """
        if self.n_tokens >= self.cap:
            raise ValueError("cache capacity exhausted")
        sched = dict(self.schedule if schedule is None else schedule)
        for l in sched:
            if not (1 <= l < self.L):
                raise ValueError("pruning layer must be in [1, L-1]")
        new_pos = self.n_tokens
        n_tot = self.n_tokens + 1
        counts = P.keep_counts(n_tot, self.L, [(l, r) for l, r in sched.items() if r < 1000])
        for l, want in (forced_selected or {}).items():       # checked before anything is written to the caches
            want = np.asarray(want, dtype=np.int64)
            if (l not in sched or want.shape[0] != counts[l] or np.any(np.diff(want) <= 0) or want[0] < 0
                    or want[-1] != new_pos):
                raise ValueError("forced selection is not valid at layer %d" % l)
        store, dtype, H, hd, d = self.store, self.dtype, self.H, self.hd, self.d
        Hkv, group = self.Hkv, self.H // self.Hkv
        selected = np.arange(n_tot, dtype=np.int64)                       # candidates of layer 0: everything
        run_pos = np.asarray([new_pos], dtype=np.int64)                   # tokens carrying a hidden state
        run_h = P._as_float(np.asarray(self.weights["embed"])[[int(token_id)]], dtype)
        res = StepResult()
        s_prev = None
        for l in range(self.L):
            if l in sched and sched[l] < 1000:
                k_keep = P.keep_count(selected.shape[0], sched[l])
                if forced_selected is not None and l in forced_selected:
                    want = np.asarray(forced_selected[l], dtype=np.int64)
                    if want.shape[0] != k_keep or not np.all(np.isin(want, selected)):
                        raise ValueError("forced selection at layer %d is not a subset of the layer below" % l)
                    selected = want
                else:
                    kept, _ = P.select_tokens(s_prev, k_keep)              # the new token is last and forced
                    selected = selected[kept]
                # tokens that carried a state out of layer l-1 but are not selected here: park the state
                dropped = ~np.isin(run_pos, selected)
                for row in np.nonzero(dropped)[0]:
                    p = int(run_pos[row])
                    assert not self.has_kv[l][p]
                    self.aux_h[l][p] = run_h[row]
                    self.has_aux[l][p] = True
            # tokens that must run this layer: selected, no K,V here yet
            need = selected[~self.has_kv[l][selected]]
            rows = np.empty((need.shape[0], d), dtype=dtype)
            carried = {int(p): i for i, p in enumerate(run_pos)}
            for i, p in enumerate(need):
                p = int(p)
                if p in carried:
                    rows[i] = run_h[carried[p]]
                else:                                                      # revived from the Aux Cache of this layer
                    if not self.has_aux[l][p]:
                        raise AssertionError("token %d has neither K,V nor an Aux Cache entry at layer %d" % (p, l))
                    rows[i] = self.aux_h[l][p]
            run_pos, run_h = need, rows
            assert run_pos.shape[0] >= 1 and run_pos[-1] == new_pos

            lw = P.LayerWeights(self.weights, l, dtype)
            m = run_pos.shape[0]
            x = P.rmsnorm(run_h, lw.attn_norm, self.eps)
            q = store(P.rope((x @ lw.wq.T).reshape(m, H, hd), run_pos, self.theta))
            k = store(P.rope((x @ lw.wk.T).reshape(m, Hkv, hd), run_pos, self.theta))
            v = store((x @ lw.wv.T).reshape(m, Hkv, hd))
            self.k[l][run_pos], self.v[l][run_pos] = k, v
            self.has_kv[l][run_pos] = True
            self.times_computed[l, run_pos] += 1
            # attention over the selected tokens, each query seeing those at or before its position
            kc, vc = self.k[l][selected], self.v[l][selected]
            visible = selected[None, :] <= run_pos[:, None]
            o = np.empty((m, H, hd), dtype=dtype)
            s = np.zeros(selected.shape[0], dtype=dtype)
            for head in range(H):
                z = (q[:, head, :] @ kc[:, head // group, :].T) / math.sqrt(hd)
                prob = P.softmax_rows(np.where(visible, z, -np.inf))
                o[:, head, :] = prob @ vc[:, head // group, :]
                s += prob[m - 1]                                           # Eq. 1: the new token's row
            s_prev = s / H
            o = store(o)
            hh = store(run_h + o.reshape(m, d) @ lw.wo.T)
            y = P.rmsnorm(hh, lw.ffn_norm, self.eps)
            a = store(P.swiglu(y, lw.w_gate, lw.w_up))
            run_h = store(hh + a @ lw.w_down.T)
            res.selected.append(selected.copy())
            res.ran.append(run_pos.copy())
            res.scores.append(s_prev)
        res.hidden_out = run_h
        xf = P.rmsnorm(run_h[-1], P._as_float(self.weights["final_norm"], dtype), self.eps)
        res.logits = P._as_float(self.weights["lm_head"], dtype) @ xf
        self.n_tokens = n_tot
        return res
