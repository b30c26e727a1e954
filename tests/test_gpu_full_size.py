"""Full-size parity: the 7B-shaped workloads in the launch configuration bench.py times.

The CPU checker cannot run 32 layers of a 7B model inside a test, so it checks what it can
compute one piece at a time: the GPU run returns every layer's input hidden states
(LAZYLLM_KEEP_HIDDEN), and for sampled layers the checker recomputes that layer from the GPU's
own input -- K, V, Eq. 1 scores, the layer output, the selection at the following pruning layer
(margin rule) and the logits from the last hidden state -- plus the properties that hold at any
size (nested kept sets, kept + aux = previous set, scores sum to one, counts)."""
import numpy as np
import pytest
import torch

from oracle import lazyllm_oracle as O
from paper_2407_14057_amd import binding as B
from paper_2407_14057_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
SHAPE = synth.LLAMA7B


@pytest.fixture(scope="module")
def model7b():
    w = synth.make_weights(SHAPE, 1002, DEV)
    model = B.Model(SHAPE.as_dict(), w, DEV)
    yield w, model
    model.close()


def _f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def _run(model, wl, flags=B.LAZYLLM_KEEP_HIDDEN):
    inp = synth.make_workload_inputs(wl)
    ids = torch.from_numpy(inp["token_ids"]).to(DEV)
    scale = None if inp["embed_scale"] is None else torch.from_numpy(inp["embed_scale"]).to(DEV)
    out = model.prefill(ids, list(wl.schedule), cu_seqlens=[int(x) for x in inp["cu_seqlens"]],
                        embed_scale=scale, flags=flags)
    torch.cuda.synchronize()
    return inp, out


def _check_structure(wl, inp, out):
    L = SHAPE.n_layers
    cu0 = inp["cu_seqlens"]
    assert out.status == 0
    for b in range(len(cu0) - 1):
        n = int(cu0[b + 1] - cu0[b])
        counts = O.keep_counts(n, L, list(wl.schedule))
        prev = np.arange(n)
        seen = set()
        for l in range(L):
            lo, hi = int(out.cu_kept(l)[b]), int(out.cu_kept(l)[b + 1])
            kept = out.kept_pos(l)[lo:hi].cpu().numpy()
            assert hi - lo == counts[l]
            assert np.all(np.diff(kept) > 0) and kept[-1] == n - 1
            if out.res.aux_pos[l]:
                alo, ahi = int(out.cu_aux(l)[b]), int(out.cu_aux(l)[b + 1])
                aux = out.aux_pos(l)[alo:ahi].cpu().numpy()
                assert np.array_equal(np.sort(np.concatenate([kept, aux])), prev)   # kept + aux = previous
                assert not (set(aux.tolist()) & seen)                               # parked at most once
                seen |= set(aux.tolist())
            else:
                assert np.array_equal(kept, prev)
            s = out.scores(l)[lo:hi].double()
            assert abs(float(s.sum()) - 1.0) < 2e-4 and float(s.min()) >= 0.0
            prev = kept
    assert sum(out.n_tokens) <= int(cu0[-1]) * L


def _check_layer(w, out, l, schedule, lo=None, hi=None, tag=""):
    """Recompute layer l from the GPU's own input and compare what the layer produced."""
    n = out.n_tokens[l]
    lo = 0 if lo is None else lo
    hi = n if hi is None else hi
    lw_bits = synth.layer_to_host_bits(w, l)
    lw = O.LayerWeights({k: [v] for k, v in lw_bits.items()}, 0, np.float64)
    h_in = _f64(out.hidden_in(l)[lo:hi])
    pos = out.kept_pos(l)[lo:hi].cpu().numpy().astype(np.int64)
    h_ref, k_ref, v_ref, s_ref = O.decoder_layer(h_in, pos, lw, SHAPE.n_heads, SHAPE.head_dim, SHAPE.rms_eps,
                                                 SHAPE.rope_theta, store=O.round_to_bf16)
    k = _f64(out.k(l)[lo:hi]); v = _f64(out.v(l)[lo:hi])
    ek = np.abs(k - k_ref).max() / np.abs(k_ref).max()
    ev = np.abs(v - v_ref).max() / np.abs(v_ref).max()
    s = out.scores(l)[lo:hi].cpu().numpy().astype(np.float64)
    es = np.abs(s / s_ref - 1.0).max()
    sched = dict(schedule)
    rep = {"layer": l, "k": float(ek), "v": float(ev), "s": float(es)}
    single = (lo == 0 and hi == n)
    if l + 1 < SHAPE.n_layers:
        if (l + 1) in sched and sched[l + 1] < 1000:
            # the selection that enters layer l+1, by the margin rule
            m = hi - lo
            kk = O.keep_count(m, sched[l + 1])
            _, decided = O.decision_margin(s_ref, kk, rel=1e-3)
            own, _ = O.select_tokens(s_ref, kk)
            want = np.zeros(m, dtype=bool); want[own] = True
            if single:
                kept_next = out.kept_pos(l + 1).cpu().numpy()
                got = np.isin(pos, kept_next)
                assert got.sum() == kk
                mism = decided & (want != got)
                rep["undecided"] = int((~decided).sum()); rep["symdiff"] = int((want != got).sum())
                assert not mism.any(), "%d decided tokens differ entering layer %d" % (int(mism.sum()), l + 1)
                # the GPU's own scores and its own selection are consistent bit for bit
                own_gpu, _ = O.select_tokens(s, kk)
                assert np.array_equal(pos[own_gpu], kept_next)
                h_next = _f64(out.hidden_in(l + 1))
                eh = np.abs(h_next - h_ref[got]).max() / np.abs(h_ref).max()
                aux = _f64(out.aux_h(l + 1))
                assert np.abs(aux - h_ref[~got]).max() / np.abs(h_ref).max() < 3e-2
                rep["h"] = float(eh)
        elif single:
            h_next = _f64(out.hidden_in(l + 1))
            rep["h"] = float(np.abs(h_next - h_ref).max() / np.abs(h_ref).max())
    elif single:
        rep["h"] = float(np.abs(_f64(out.hidden_out) - h_ref).max() / np.abs(h_ref).max())
    print(tag, rep, flush=True)
    assert ek < 2e-2 and ev < 2e-2, rep
    assert es < 2e-2, rep
    assert rep.get("h", 0.0) < 3e-2, rep
    return rep


def _check_logits(w, out, b=0):
    L = SHAPE.n_layers
    last_row = int(out.cu_kept(L - 1)[b + 1]) - 1
    h_last = _f64(out.hidden_out[last_row])
    g = _f64(w["final_norm"]); wl = _f64(w["lm_head"])
    ref = wl @ O.rmsnorm(h_last, g, SHAPE.rms_eps)
    got = out.logits[b].cpu().numpy().astype(np.float64)
    err = np.abs(got - ref).max() / (ref.max() - ref.min())
    print("logits err/range", err, flush=True)
    assert err <= 2e-2


def test_headline_3376(model7b):
    w, model = model7b
    wl = synth.WORKLOADS["7b_3376"]
    inp, out = _run(model, wl)
    assert sorted(set(out.n_tokens), reverse=True) == [3376, 2364, 1182, 355]
    _check_structure(wl, inp, out)
    for l in (0, 7, 8, 15, 23, 31):
        _check_layer(w, out, l, wl.schedule, tag="7b_3376")
    _check_logits(w, out)
    # the timed configuration (no hidden-state copies) returns the same bits
    snap = (out.logits.clone(), out.kept_pos(31).clone(), out.k(31).clone())
    _, out2 = _run(model, wl, flags=0)
    assert torch.equal(snap[0], out2.logits) and torch.equal(snap[1], out2.kept_pos(31))
    assert torch.equal(snap[2], out2.k(31))


def test_needles_3376(model7b):
    w, model = model7b
    wl = synth.WORKLOADS["7b_3376_needles"]
    inp, out = _run(model, wl)
    assert sorted(set(out.n_tokens), reverse=True) == [3376, 1688, 844, 422]
    _check_structure(wl, inp, out)
    # layer 0 input is the scaled embedding, exactly
    ids = inp["token_ids"]
    emb = w["embed"][torch.from_numpy(ids).to(DEV).long()].float() * torch.from_numpy(inp["embed_scale"]).to(DEV)[:, None]
    assert torch.equal(out.hidden_in(0), emb.to(torch.bfloat16))
    for l in (3, 11, 19):
        _check_layer(w, out, l, wl.schedule, tag="needles")
    _check_logits(w, out)
    # how heavy-tailed the scores are that selection sees (reported, not asserted)
    for l in (3, 11, 19):
        s = np.sort(out.scores(l).cpu().numpy().astype(np.float64))[::-1]
        print("needles layer %d: top-64 mass %.3f, max/median %.1f" % (l, s[:64].sum(), s[0] / np.median(s)), flush=True)


def test_long_8192(model7b):
    w, model = model7b
    wl = synth.WORKLOADS["7b_8192"]
    inp, out = _run(model, wl)
    assert sorted(set(out.n_tokens), reverse=True) == [8192, 4916, 1967, 394]
    _check_structure(wl, inp, out)
    for l in (15, 23, 31):                      # 4916-, 1967- and 394-token layers
        _check_layer(w, out, l, wl.schedule, tag="7b_8192")
    _check_logits(w, out)


def test_batch8(model7b):
    w, model = model7b
    wl = synth.WORKLOADS["7b_batch8"]
    inp, out = _run(model, wl)
    _check_structure(wl, inp, out)
    # one sequence of the packed batch, at a layer after two prunings, against the checker
    b = int(np.argmin(np.asarray(wl.seqlens)))
    l = 16
    lo, hi = int(out.cu_kept(l)[b]), int(out.cu_kept(l)[b + 1])
    _check_layer(w, out, l, wl.schedule, lo=lo, hi=hi, tag="batch8 seq %d" % b)
    for bb in (0, 7):
        _check_logits(w, out, bb)
