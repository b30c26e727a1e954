"""Pins for the CPU checker's whole prefill: a library transformer for the dense
path and Eq. 1, closed forms, and the structural facts the paper states
(nested kept sets, Aux Cache completeness, each token computed at most once
per layer, cumulative usage bounded by the baseline)."""
import dataclasses
import os

import numpy as np
import pytest
import torch

from oracle import lazyllm_oracle as O
from paper_2407_14057_amd import synth

SMALL = dataclasses.replace(synth.TINY, vocab=256)


def _weights(shape, seed=11, jitter=0.25):
    return synth.weights_to_host_bits(synth.make_weights(shape, seed, "cpu", gain_jitter=jitter))


def _hf_model(shape, wb):
    from transformers import LlamaConfig, LlamaForCausalLM
    cfg = LlamaConfig(vocab_size=shape.vocab, hidden_size=shape.d_model, intermediate_size=shape.d_ffn,
                      num_hidden_layers=shape.n_layers, num_attention_heads=shape.n_heads,
                      num_key_value_heads=shape.n_heads, rms_norm_eps=shape.rms_eps,
                      rope_theta=shape.rope_theta, max_position_embeddings=4096,
                      attn_implementation="eager", tie_word_embeddings=False, attention_bias=False,
                      mlp_bias=False)
    model = LlamaForCausalLM(cfg).eval().double()
    f = lambda bits: torch.from_numpy(O.bf16_bits_to_float(bits, np.float64))
    sd = {"model.embed_tokens.weight": f(wb["embed"]), "model.norm.weight": f(wb["final_norm"]),
          "lm_head.weight": f(wb["lm_head"])}
    names = {"attn_norm": "input_layernorm", "ffn_norm": "post_attention_layernorm",
             "wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj",
             "wo": "self_attn.o_proj", "w_gate": "mlp.gate_proj", "w_up": "mlp.up_proj",
             "w_down": "mlp.down_proj"}
    for l in range(shape.n_layers):
        for mine, theirs in names.items():
            sd[f"model.layers.{l}.{theirs}.weight"] = f(wb[mine][l])
    missing, unexpected = model.load_state_dict(sd, strict=False)
    assert not [m for m in missing if "rotary" not in m] and not unexpected
    return model


def test_dense_prefill_matches_library_transformer():
    """Unpruned path, hidden states, K/V and Eq. 1 against HF's Llama (eager attention, fp64)."""
    wb = _weights(SMALL)
    ids = synth.make_prompt(96, SMALL.vocab, 5)
    res = O.prefill(SMALL.as_dict(), wb, ids, [], keep_hidden=True)
    model = _hf_model(SMALL, wb)
    with torch.no_grad():
        out = model(torch.from_numpy(ids.astype(np.int64))[None], output_attentions=True,
                    output_hidden_states=True, use_cache=True)
    # the library forms its rotary angles in fp32, which bounds the agreement near 1e-7
    tol = 2e-6
    assert np.allclose(res.logits, out.logits[0, -1].numpy(), atol=tol)
    for l in range(SMALL.n_layers):
        assert np.allclose(res.hidden_in[l], out.hidden_states[l][0].numpy(), atol=tol)
        A = out.attentions[l][0].numpy()                       # [H, query, key]
        assert np.allclose(res.scores[l], A[:, -1, :].mean(0), atol=1e-8)       # Eq. 1
        kc, vc = out.past_key_values.layers[l].keys, out.past_key_values.layers[l].values
        assert np.allclose(res.k[l], kc[0].permute(1, 0, 2).numpy(), atol=2e-5)  # post-RoPE keys
        assert np.allclose(res.v[l], vc[0].permute(1, 0, 2).numpy(), atol=tol)
    # mistakes this must catch: a dropped gain, a wrong RoPE pairing, a transposed weight
    assert float(np.abs(res.logits).max()) > 0.05


def test_zeroed_output_projections_leave_the_embedding():
    wb = _weights(SMALL)
    for l in range(SMALL.n_layers):
        wb["wo"][l] = np.zeros_like(wb["wo"][l])
        wb["w_down"][l] = np.zeros_like(wb["w_down"][l])
    ids = synth.make_prompt(40, SMALL.vocab, 6)
    res = O.prefill(SMALL.as_dict(), wb, ids, [(2, 500)])
    e = O.bf16_bits_to_float(wb["embed"][ids[-1]])
    g = O.bf16_bits_to_float(wb["final_norm"])
    x = torch.nn.functional.rms_norm(torch.from_numpy(e), (SMALL.d_model,), torch.from_numpy(g), SMALL.rms_eps)
    ref = torch.from_numpy(O.bf16_bits_to_float(wb["lm_head"])) @ x
    assert np.allclose(res.logits, ref.numpy(), atol=1e-12)
    # and every Aux Cache row is the untouched embedding of the dropped token
    E = O.bf16_bits_to_float(wb["embed"])
    assert np.array_equal(res.aux_h[2], E[ids[res.aux_pos[2]]])


def test_single_token_prompt():
    wb = _weights(SMALL)
    res = O.prefill(SMALL.as_dict(), wb, np.array([7], np.int32), [])
    assert all(np.array_equal(s, [1.0]) for s in res.scores)
    assert all(list(p) == [0] for p in res.kept_pos)


def test_zero_query_weights_give_uniform_scores():
    wb = _weights(SMALL)
    for l in range(SMALL.n_layers):
        wb["wq"][l] = np.zeros_like(wb["wq"][l])
    res = O.prefill(SMALL.as_dict(), wb, synth.make_prompt(33, SMALL.vocab, 8), [])
    for s in res.scores:
        assert np.allclose(s, 1.0 / 33, atol=1e-15)
    # all-equal scores: pruning then keeps the lowest indices and the last token
    res = O.prefill(SMALL.as_dict(), wb, synth.make_prompt(33, SMALL.vocab, 8), [(1, 500)])
    assert list(res.kept_pos[1]) == list(range(16)) + [32]


def test_keep_everything_is_dense_prefill_bit_for_bit():
    wb = _weights(SMALL)
    ids = synth.make_prompt(64, SMALL.vocab, 9)
    a = O.prefill(SMALL.as_dict(), wb, ids, [])
    b = O.prefill(SMALL.as_dict(), wb, ids, [(1, 1000), (3, 1000)])
    assert np.array_equal(a.logits, b.logits)
    assert all(np.array_equal(x, y) for x, y in zip(a.k, b.k))
    assert not b.aux_pos


@pytest.mark.parametrize("bf16_storage", [False, True])
def test_pruned_prefill_structure(bf16_storage):
    wb = _weights(SMALL)
    N = 200
    ids = synth.make_prompt(N, SMALL.vocab, 10)
    sched = [(1, 800), (2, 700), (3, 500)]
    res = O.prefill(SMALL.as_dict(), wb, ids, sched, bf16_storage=bf16_storage, keep_hidden=True)
    counts = O.keep_counts(N, SMALL.n_layers, sched)
    assert counts == [200, 160, 112, 56]
    prev = np.arange(N)
    seen_aux = set()
    for l in range(SMALL.n_layers):
        kept = res.kept_pos[l]
        assert len(kept) == counts[l] == res.k[l].shape[0] == res.scores[l].shape[0]
        assert np.all(np.diff(kept) > 0) and kept[-1] == N - 1            # ascending, last token kept
        assert set(kept) <= set(prev)                                      # nested
        if l in res.aux_pos:
            aux = res.aux_pos[l]
            assert sorted(list(kept) + list(aux)) == list(prev)            # kept + aux = previous set
            assert not (set(aux) & seen_aux)                               # parked at most once
            seen_aux |= set(aux)
            # parked hidden state = the dropped token's input to this layer = output of layer l-1
            assert res.aux_h[l].shape == (len(aux), SMALL.d_model)
        assert abs(res.scores[l].sum() - 1.0) < (1e-12 if not bf16_storage else 1e-9)
        prev = kept
    assert sum(counts) <= N * SMALL.n_layers                               # bounded by the baseline
    # the set chosen at layer l is the top of layer l-1's scores
    k_idx, _ = O.select_tokens(res.scores[1], counts[2])
    assert np.array_equal(res.kept_pos[2], res.kept_pos[1][k_idx])


def test_pruning_equals_dense_layers_on_the_subsequence():
    """From a pruning layer on, the run is a dense transformer on the kept rows with
    their original position ids."""
    wb = _weights(SMALL)
    sd = SMALL.as_dict()
    ids = synth.make_prompt(120, SMALL.vocab, 12)
    res = O.prefill(sd, wb, ids, [(2, 400)], keep_hidden=True)
    dense = O.prefill(sd, wb, ids, [], keep_hidden=True)
    kept = res.kept_pos[2]
    h = dense.hidden_in[2][kept]                      # dense and pruned agree up to layer 1
    assert np.array_equal(h, res.hidden_in[2])
    aux_rows = dense.hidden_in[2][res.aux_pos[2]]
    assert np.array_equal(aux_rows, res.aux_h[2])
    for l in (2, 3):
        lw = O.LayerWeights(wb, l, np.float64)
        h, k, v, s = O.decoder_layer(h, kept, lw, SMALL.n_heads, SMALL.head_dim, SMALL.rms_eps, SMALL.rope_theta)
        assert np.array_equal(k, res.k[l]) and np.array_equal(s, res.scores[l])
    assert np.array_equal(h, res.hidden_out)
    # original positions matter: renumbering 0..k-1 changes the keys
    lw = O.LayerWeights(wb, 2, np.float64)
    _, k2, _, _ = O.decoder_layer(res.hidden_in[2], np.arange(len(kept)), lw, SMALL.n_heads,
                                  SMALL.head_dim, SMALL.rms_eps, SMALL.rope_theta)
    assert not np.allclose(k2, res.k[2])


def test_keeping_one_token_makes_attention_the_identity_on_v():
    wb = _weights(SMALL)
    ids = synth.make_prompt(30, SMALL.vocab, 13)
    res = O.prefill(SMALL.as_dict(), wb, ids, [(2, 1)], keep_hidden=True)
    assert list(res.kept_pos[2]) == [29] and list(res.kept_pos[3]) == [29]
    assert np.array_equal(res.scores[2], [1.0]) and np.array_equal(res.scores[3], [1.0])
    assert len(res.aux_pos[2]) == 29
    # with one token, the attention output is v itself: h_mid = h + Wo v
    lw = O.LayerWeights(wb, 2, np.float64)
    h = res.hidden_in[2]
    h_mid = h + res.v[2].reshape(1, -1) @ lw.wo.T
    y = O.rmsnorm(h_mid, lw.ffn_norm, SMALL.rms_eps)
    h_out = h_mid + O.swiglu(y, lw.w_gate, lw.w_up) @ lw.w_down.T
    assert np.allclose(h_out, res.hidden_in[3], atol=1e-13)


def test_forced_keep_and_validation():
    wb = _weights(SMALL)
    sd = SMALL.as_dict()
    ids = synth.make_prompt(50, SMALL.vocab, 14)
    sched = [(1, 600), (3, 500)]
    a = O.prefill(sd, wb, ids, sched)
    b = O.prefill(sd, wb, ids, sched, forced_keep={1: a.kept_pos[1], 3: a.kept_pos[3]})
    assert np.array_equal(a.logits, b.logits)
    other = a.kept_pos[1].copy()
    dropped = a.aux_pos[1][0]
    other[0] = dropped
    other.sort()
    c = O.prefill(sd, wb, ids, sched, forced_keep={1: other})
    assert dropped in c.kept_pos[1] and not np.array_equal(c.logits, a.logits)
    with pytest.raises(ValueError):
        O.prefill(sd, wb, ids, sched, forced_keep={1: a.kept_pos[1][:-1]})       # wrong count
    with pytest.raises(ValueError):
        O.prefill(sd, wb, ids, sched, forced_keep={3: np.arange(15)})            # not a subset / no last
    with pytest.raises(ValueError):
        O.prefill(sd, wb, ids, [(0, 500)])                                       # layer 0 cannot prune


def test_embed_scale_and_batch():
    wb = _weights(SMALL)
    sd = SMALL.as_dict()
    ids = synth.make_prompt(70, SMALL.vocab, 15)
    scale = synth.make_needle_scale(40, 5, 3)
    cu = np.array([0, 40, 70], np.int32)
    full_scale = np.concatenate([scale, np.ones(30, np.float32)])
    rs = O.prefill_batch(sd, wb, ids, cu, [(2, 500)], embed_scale=full_scale)
    r0 = O.prefill(sd, wb, ids[:40], [(2, 500)], embed_scale=scale)
    r1 = O.prefill(sd, wb, ids[40:], [(2, 500)])
    assert np.array_equal(rs[0].logits, r0.logits) and np.array_equal(rs[1].logits, r1.logits)
    # the scale multiplies the embedding row and nothing else
    r0u = O.prefill(sd, wb, ids[:40], [(2, 500)], keep_hidden=True)
    r0s = O.prefill(sd, wb, ids[:40], [(2, 500)], embed_scale=scale, keep_hidden=True)
    assert np.array_equal(r0s.hidden_in[0], r0u.hidden_in[0] * scale[:, None].astype(np.float64))


def test_fp32_variant_tracks_fp64():
    wb = _weights(SMALL)
    ids = synth.make_prompt(64, SMALL.vocab, 16)
    a = O.prefill(SMALL.as_dict(), wb, ids, [(2, 500)])
    b = O.prefill(SMALL.as_dict(), wb, ids, [(2, 500)], dtype=np.float32, forced_keep={2: a.kept_pos[2]})
    assert b.logits.dtype == np.float32
    assert np.allclose(a.logits, b.logits, atol=2e-5)


def test_tiny512_regression_fixture():
    """The checker still computes what tests/golden/make_golden.py froze (a later edit of its
    arithmetic must show up here and name, in its commit, the passage that justifies it)."""
    import json
    import importlib.util
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    got = mod.compute()
    with open(os.path.join(here, "golden", "tiny512_oracle.json")) as f:
        want = json.load(f)
    for key in ("n_per_layer", "kept_pos_sha256", "kept_pos_layer3_head", "aux_counts", "logits_argmax"):
        assert got[key] == want[key], key
    assert want["n_per_layer"] == [512, 512, 359, 180]
    for key in ("scores_layer1_first8", "scores_layer3_last4", "logits_first8"):
        assert np.allclose(got[key], want[key], rtol=1e-9, atol=1e-12), key
    assert abs(got["logits_sum"] - want["logits_sum"]) < 1e-7


def test_grouped_query_attention_matches_library_transformer():
    """Model variant with fewer K,V heads than query heads: hidden states, K/V and Eq. 1 (the mean
    over ALL query heads' maps) against HF's Llama with num_key_value_heads below the head count."""
    shape = dataclasses.replace(SMALL, n_kv_heads=2)
    wb = _weights(shape, seed=17)
    assert wb["wk"][0].shape == (2 * shape.head_dim, shape.d_model)
    ids = synth.make_prompt(80, shape.vocab, 6)
    res = O.prefill(shape.as_dict(), wb, ids, [], keep_hidden=True)
    from transformers import LlamaConfig, LlamaForCausalLM
    cfg = LlamaConfig(vocab_size=shape.vocab, hidden_size=shape.d_model, intermediate_size=shape.d_ffn,
                      num_hidden_layers=shape.n_layers, num_attention_heads=shape.n_heads,
                      num_key_value_heads=2, rms_norm_eps=shape.rms_eps, rope_theta=shape.rope_theta,
                      max_position_embeddings=4096, attn_implementation="eager", tie_word_embeddings=False,
                      attention_bias=False, mlp_bias=False)
    model = LlamaForCausalLM(cfg).eval().double()
    f = lambda bits: torch.from_numpy(O.bf16_bits_to_float(bits, np.float64))
    sd = {"model.embed_tokens.weight": f(wb["embed"]), "model.norm.weight": f(wb["final_norm"]),
          "lm_head.weight": f(wb["lm_head"])}
    names = {"attn_norm": "input_layernorm", "ffn_norm": "post_attention_layernorm",
             "wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj",
             "wo": "self_attn.o_proj", "w_gate": "mlp.gate_proj", "w_up": "mlp.up_proj",
             "w_down": "mlp.down_proj"}
    for l in range(shape.n_layers):
        for mine, theirs in names.items():
            sd[f"model.layers.{l}.{theirs}.weight"] = f(wb[mine][l])
    missing, unexpected = model.load_state_dict(sd, strict=False)
    assert not [m for m in missing if "rotary" not in m] and not unexpected
    with torch.no_grad():
        out = model(torch.from_numpy(ids.astype(np.int64))[None], output_attentions=True,
                    output_hidden_states=True, use_cache=True)
    tol = 2e-6
    assert np.allclose(res.logits, out.logits[0, -1].numpy(), atol=tol)
    for l in range(shape.n_layers):
        assert np.allclose(res.hidden_in[l], out.hidden_states[l][0].numpy(), atol=tol)
        A = out.attentions[l][0].numpy()                       # [H, query, key]
        assert A.shape[0] == shape.n_heads
        assert np.allclose(res.scores[l], A[:, -1, :].mean(axis=0), atol=tol)
        assert res.k[l].shape == (80, 2, shape.head_dim)


def test_grouped_query_pruned_prefill_and_decoding_keep_their_structure():
    from oracle import lazyllm_decode_oracle as D
    shape = dataclasses.replace(SMALL, n_kv_heads=1)
    wb = _weights(shape, seed=19)
    ids = synth.make_prompt(60, shape.vocab, 8)
    sched = [(1, 700), (3, 500)]
    res = O.prefill(shape.as_dict(), wb, ids, sched)
    assert [len(p) for p in res.kept_pos] == O.keep_counts(60, shape.n_layers, sched)
    # with one K,V head shared by all query heads the dense step still equals the longer prefill
    dense = O.prefill(shape.as_dict(), wb, ids, [])
    gen = D.Generation(shape.as_dict(), wb, [], dense, 60, 62)
    out = gen.step(5)
    full = O.prefill(shape.as_dict(), wb, np.concatenate([ids, [5]]), [])
    assert np.allclose(out.logits, full.logits, atol=1e-10)
    gen2 = D.Generation(shape.as_dict(), wb, sched, res, 60, 63)
    for tok in (1, 2, 3):
        o2 = gen2.step(tok)
        assert all(abs(s.sum() - 1) < 1e-12 for s in o2.scores)
    assert gen2.times_computed.max() == 1


# ---------------------------------------------------------------- bf16-storage rounding points

def _recording_store(log):
    def store(t):
        log.append(np.array(t, copy=True))
        return t
    return store


def test_storage_mode_rounds_exactly_the_tensors_the_data_flow_writes():
    """The bf16-storage mode models stores to bf16 tensors: per layer v, q (after the rotary
    embedding), k (after it), the attention output o, h after the attention block, the SwiGLU
    output a, h after the MLP block -- in that order, each once -- and NOT the normalised
    activations x, y (RMSNorm is folded into the projections that consume it, so they are never
    written).  A rounding point added, dropped, moved or reordered fails here."""
    shape = SMALL
    wb = _weights(shape)
    H, hd, d, f = shape.n_heads, shape.head_dim, shape.d_model, shape.d_ffn
    m = 37
    rng = np.random.default_rng(3)
    h = rng.standard_normal((m, d))
    pos = np.sort(rng.choice(500, m, replace=False)).astype(np.int64)
    lw = O.LayerWeights(wb, 1, np.float64)
    log = []
    h_out, k, v, s = O.decoder_layer(h, pos, lw, H, hd, shape.rms_eps, shape.rope_theta, store=_recording_store(log))
    assert [t.shape for t in log] == [(m, H, hd), (m, H, hd), (m, H, hd), (m, H, hd), (m, d), (m, f), (m, d)]
    # what each store receives, from the layer equations written out with library routines
    rms = lambda t, g: torch.nn.functional.rms_norm(torch.from_numpy(t), (d,), torch.from_numpy(g), shape.rms_eps).numpy()
    x = rms(h, lw.attn_norm)
    assert np.allclose(log[0], (x @ lw.wv.T).reshape(m, H, hd), atol=1e-12)                     # v, unrotated
    assert np.allclose(log[1], O.rope((x @ lw.wq.T).reshape(m, H, hd), pos, shape.rope_theta), atol=1e-12)
    assert np.allclose(log[2], O.rope((x @ lw.wk.T).reshape(m, H, hd), pos, shape.rope_theta), atol=1e-12)
    sdpa = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(log[1]).permute(1, 0, 2)[None], torch.from_numpy(log[2]).permute(1, 0, 2)[None],
        torch.from_numpy(log[0]).permute(1, 0, 2)[None], is_causal=True)[0].permute(1, 0, 2).numpy()
    assert np.allclose(log[3], sdpa, atol=1e-12)                                               # o
    h1 = h + log[3].reshape(m, d) @ lw.wo.T
    assert np.allclose(log[4], h1, atol=1e-12)                                                 # h after attention
    y = rms(h1, lw.ffn_norm)
    a = torch.nn.functional.silu(torch.from_numpy(y @ lw.w_gate.T)).numpy() * (y @ lw.w_up.T)
    assert np.allclose(log[5], a, atol=1e-12)                                                  # SwiGLU output
    assert np.allclose(log[6], h1 + a @ lw.w_down.T, atol=1e-12)                               # h after the MLP
    assert np.array_equal(log[6], h_out) and np.array_equal(log[2], k) and np.array_equal(log[0], v)
    # neither normalised activation is ever handed to store
    for t in log:
        assert t.shape != (m, d) or (not np.allclose(t, x) and not np.allclose(t, y))


def test_storage_mode_identity_is_the_plain_path_and_rounding_is_real():
    shape = SMALL
    wb = _weights(shape)
    ids = synth.make_prompt(64, shape.vocab, 8)
    sched = [(1, 700), (3, 500)]
    plain = O.prefill(shape.as_dict(), wb, ids, sched)
    ident = O.prefill(shape.as_dict(), wb, ids, sched, bf16_storage=False)
    assert np.array_equal(plain.logits, ident.logits)
    # decoder_layer with an explicit identity store: bit for bit the default
    lw = O.LayerWeights(wb, 0, np.float64)
    h = np.random.default_rng(5).standard_normal((20, shape.d_model))
    pos = np.arange(20, dtype=np.int64)
    a = O.decoder_layer(h, pos, lw, shape.n_heads, shape.head_dim, shape.rms_eps, shape.rope_theta)
    b = O.decoder_layer(h, pos, lw, shape.n_heads, shape.head_dim, shape.rms_eps, shape.rope_theta, store=lambda t: t)
    assert all(np.array_equal(u, w_) for u, w_ in zip(a, b))
    # with bf16 storage every returned tensor is a bf16 value, and the result differs from fp64
    r = O.prefill(shape.as_dict(), wb, ids, sched, bf16_storage=True, keep_hidden=True)
    for l in range(shape.n_layers):
        for t in (r.k[l], r.v[l]) + ((r.hidden_in[l],) if l > 0 else ()):
            assert np.array_equal(t, O.round_to_bf16(t))
    assert np.array_equal(r.hidden_out, O.round_to_bf16(r.hidden_out))
    assert not np.array_equal(r.logits, plain.logits)
    # the embedding rows are bf16 already: without a per-token scale nothing is rounded before layer 0,
    # with one the scaled row is (it is what the embedding step writes)
    scale = np.full(64, 3.0, dtype=np.float32); scale[5] = 1.0 / 3.0
    rs = O.prefill(shape.as_dict(), wb, ids, [], bf16_storage=True, embed_scale=scale, keep_hidden=True, n_layers=1)
    e = O.bf16_bits_to_float(wb["embed"][ids]) * scale[:, None].astype(np.float64)
    assert np.array_equal(rs.hidden_in[0], O.round_to_bf16(e)) and not np.array_equal(rs.hidden_in[0], e)
