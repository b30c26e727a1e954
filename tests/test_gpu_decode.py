"""Parity of the decoding steps with Aux Cache revival, through the C ABI, against the CPU checker.

Both sides start from the same pruned prefill (the checker is fed the GPU's kept sets) and are
fed the same token at every step.  Per step and pruning layer the GPU's selection must agree
with the checker's own scores of the layer below on every token further than 1e-3 (relative)
from the threshold; the checker then continues with the GPU's selection, and everything
downstream is compared: which tokens ran each layer (exact), Eq. 1 scores, logits
(<= 2e-2 of the checker's logit range, against the fp64 checker), and the caches (presence
tables exact; K, V and Aux Cache rows against the checker run with bf16 storage)."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import lazyllm_decode_oracle as D
from oracle import lazyllm_oracle as O
from paper_2407_14057_amd import binding as B
from paper_2407_14057_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
HD128 = dataclasses.replace(synth.TINY, n_heads=2, head_dim=128)


def _to_dev(w):
    return {k: ([t.to(DEV) for t in v] if isinstance(v, list) else v.to(DEV)) for k, v in w.items()}


def _model(shape, seed, jitter=0.0, std=0.02):
    w = synth.make_weights(shape, seed, "cpu", std=std, gain_jitter=jitter)
    return synth.weights_to_host_bits(w), B.Model(shape.as_dict(), _to_dev(w), DEV)


@pytest.fixture(scope="module")
def tiny():
    wb, model = _model(synth.TINY, 1001)
    yield synth.TINY, wb, model
    model.close()


@pytest.fixture(scope="module")
def tiny_wide():
    """Larger weights: attention logits of order 1 instead of 0.1, far from uniform."""
    wb, model = _model(synth.TINY, 1021, jitter=0.3, std=0.05)
    yield synth.TINY, wb, model
    model.close()


@pytest.fixture(scope="module")
def hd128():
    wb, model = _model(HD128, 1031, jitter=0.2)
    yield HD128, wb, model
    model.close()


def _f(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def _check_caches(shape, view, g16, n_tot, prune_layers, kv_tol=3e-2, aux_tol=0.05):
    L, d = shape.n_layers, shape.d_model
    worst = 0.0
    for l in range(L):
        has = view["has_kv"][l].cpu().numpy().astype(bool)
        assert np.array_equal(has[:n_tot], g16.has_kv[l][:n_tot]), "K,V presence differs at layer %d" % l
        assert not has[n_tot:].any()
        idx = np.nonzero(has)[0]
        k = _f(view["k"][l])[idx]
        v = _f(view["vt"][l]).T[idx]
        rk, rv = g16.k[l][idx].reshape(len(idx), -1), g16.v[l][idx].reshape(len(idx), -1)
        worst = max(worst, np.abs(k - rk).max() / max(np.abs(rk).max(), 1e-9),
                    np.abs(v - rv).max() / max(np.abs(rv).max(), 1e-9))
        # rows without K,V were never written
        gone = np.nonzero(~has)[0]
        assert not _f(view["k"][l])[gone].any() and not _f(view["vt"][l]).T[gone].any()
        if l in prune_layers:
            ha = view["has_aux"][l].cpu().numpy().astype(bool)
            assert np.array_equal(ha[:n_tot], g16.has_aux[l][:n_tot]), "Aux Cache presence differs at layer %d" % l
            ia = np.nonzero(ha)[0]
            if len(ia):
                a, ra = _f(view["aux_h"][l])[ia], g16.aux_h[l][ia]
                assert np.abs(a - ra).max() <= aux_tol * max(1.0, np.abs(ra).max())
        else:
            assert view["aux_h"][l] is None
    assert worst < kv_tol, worst
    return worst


def run_case(shape, wb, model, ids, schedule, new_tokens, extra=3, label="", band=1e-3, s_tol=(2e-2, 5e-2),
             gemm8=False, logit_tol=2e-2, kv_tol=3e-2, aux_tol=0.05):
    """gemm8: the model's prefill ran its projections in the 8-bit variant and so does the checker's;
    the decoding steps are 16-bit on both sides."""
    sd, L = shape.as_dict(), shape.n_layers
    ids = np.asarray(ids)
    out = model.prefill(torch.from_numpy(ids.astype(np.int32)).to(DEV), schedule)
    torch.cuda.synchronize()
    assert out.status == 0
    prune_layers = [l for l, p in schedule if p < 1000]
    forced = {p: out.kept_pos(p).cpu().numpy().astype(np.int64) for p in prune_layers}
    ref16 = O.prefill(sd, wb, ids, schedule, bf16_storage=True, forced_keep=forced, gemm8=gemm8)
    ref64 = O.prefill(sd, wb, ids, schedule, forced_keep=forced, gemm8=gemm8)
    cap = len(ids) + len(new_tokens) + extra
    gen = B.Generation(model, schedule, out, cap)
    g16 = D.Generation(sd, wb, schedule, ref16, len(ids), cap, bf16_storage=True)
    g64 = D.Generation(sd, wb, schedule, ref64, len(ids), cap)
    torch.cuda.synchronize()
    # the state right after it is made: the prefill's rows, bit for bit, at their positions
    view = gen.view()
    for l in range(L):
        pos = out.kept_pos(l).long()
        assert torch.equal(view["k"][l][pos], out.k(l).reshape(len(pos), -1))
        assert torch.equal(view["vt"][l].t()[pos], out.v(l).reshape(len(pos), -1))
    _check_caches(shape, view, g16, len(ids), prune_layers, kv_tol, aux_tol)

    report = {"revived": [], "undecided": 0, "logit_err": 0.0, "s16": 0.0, "s64": 0.0}
    for t, tok in enumerate(new_tokens):
        n_tot = len(ids) + t + 1
        so = gen.step(torch.tensor([int(tok)], dtype=torch.int32, device=DEV))
        torch.cuda.synchronize()
        assert so.status == 0 and so.n_tokens == n_tot and so.position == n_tot - 1
        sel = []
        for l in range(L):
            m = so.selected(l)
            sel.append(np.arange(n_tot) if m is None else np.nonzero(m.cpu().numpy())[0])
        forced_sel = {p: sel[p] for p in prune_layers}
        r16 = g16.step(int(tok), forced_selected=forced_sel)
        r64 = g64.step(int(tok), forced_selected=forced_sel)
        counts = O.keep_counts(n_tot, L, schedule)
        for l in range(L):
            assert len(sel[l]) == counts[l] == so.n_selected[l]
            assert np.array_equal(sel[l], r16.selected[l])
            if l in prune_layers:
                s_prev = r16.scores[l - 1]
                tau, decided = O.decision_margin(s_prev, counts[l], rel=band)
                own, _ = O.select_tokens(s_prev, counts[l])
                want = np.zeros(len(s_prev), dtype=bool)
                want[own] = True
                got = np.isin(r16.selected[l - 1], sel[l])
                mism = decided & (want != got)
                assert not mism.any(), "step %d layer %d: %d decided tokens differ" % (t, l, int(mism.sum()))
                report["undecided"] += int((~decided).sum())
            assert so.n_ran[l] == len(r16.ran[l])
            assert np.array_equal(so.ran_pos(l).cpu().numpy(), r16.ran[l]), "step %d layer %d" % (t, l)
            s = so.scores(l).cpu().numpy().astype(np.float64)
            assert abs(s.sum() - 1.0) < 1e-4
            outside = np.ones(n_tot, dtype=bool)
            outside[sel[l]] = False
            assert not s[outside].any()
            report["s16"] = max(report["s16"], float(np.abs(s[sel[l]] / r16.scores[l] - 1).max()))
            report["s64"] = max(report["s64"], float(np.abs(s[sel[l]] / r64.scores[l] - 1).max()))
        report["revived"].append([int(n) - 1 for n in so.n_ran])
        logits = so.logits.cpu().numpy().astype(np.float64)
        rng_ = r64.logits.max() - r64.logits.min()
        report["logit_err"] = max(report["logit_err"], float(np.abs(logits - r64.logits).max() / rng_))
        _check_caches(shape, gen.view(), g16, n_tot, prune_layers, kv_tol, aux_tol)
    print(label, report)
    assert report["s16"] < s_tol[0] and report["s64"] < s_tol[1], report
    assert report["logit_err"] <= logit_tol, report
    gen.close()
    return report


def test_tiny_decode_matches_checker(tiny):
    shape, wb, model = tiny
    ids = synth.make_prompt(200, shape.vocab, 71)
    rep = run_case(shape, wb, model, ids, [(2, 700), (3, 500)], [5, 900, 33, 512, 7], label="tiny")
    assert sum(sum(r) for r in rep["revived"]) > 0            # the revival path was exercised


def test_selections_that_move(tiny_wide):
    shape, wb, model = tiny_wide
    ids = synth.make_prompt(333, shape.vocab, 72)
    # With logits of order 1 the bf16 rounding of q, k and of the probabilities moves a score by up
    # to ~1e-2 relative (the standard-deviation-0.02 models used elsewhere: 1e-3), so the band in
    # which a selection may differ is widened accordingly for this stress model.
    rep = run_case(shape, wb, model, ids, [(1, 600), (2, 500), (3, 400)], [1, 2, 3, 1000, 4, 77, 78, 79],
                   label="moving", band=3e-2, s_tol=(5e-2, 1e-1))
    assert sum(sum(r) for r in rep["revived"]) > 0


def test_head_dim_128(hd128):
    shape, wb, model = hd128
    ids = synth.make_prompt(150, shape.vocab, 73)
    run_case(shape, wb, model, ids, [(1, 800), (3, 300)], [9, 8, 7, 6], label="hd128")


@pytest.mark.parametrize("base,kv", [(synth.TINY, 2), (HD128, 1)])
def test_shared_kv_heads(base, kv):
    """Grouped-query variant: K,V heads shared by groups of query heads (caches half as wide)."""
    shape = dataclasses.replace(base, n_kv_heads=kv)
    wb, model = _model(shape, 1041 + kv, jitter=0.2)
    ids = synth.make_prompt(210, shape.vocab, 77)
    rep = run_case(shape, wb, model, ids, [(1, 700), (3, 400)], [3, 1000, 17, 4], label="gqa %d" % kv)
    assert sum(sum(r) for r in rep["revived"]) > 0
    model.close()


def test_dense_schedule_never_revives(tiny):
    shape, wb, model = tiny
    ids = synth.make_prompt(129, shape.vocab, 74)
    rep = run_case(shape, wb, model, ids, [], [3, 4, 5], label="dense")
    assert all(all(x == 0 for x in r) for r in rep["revived"])


@pytest.mark.parametrize("n,sched", [(1, []), (2, [(1, 500)]), (64, [(3, 1)]), (65, [(1, 900), (2, 500), (3, 100)])])
def test_edge_shapes(tiny, n, sched):
    shape, wb, model = tiny
    ids = synth.make_prompt(n, shape.vocab, 500 + n)
    run_case(shape, wb, model, ids, sched, [11, 12, 13], extra=1, label="n=%d %s" % (n, sched))


def test_capacity_and_argument_checks(tiny):
    shape, wb, model = tiny
    ids = synth.make_prompt(40, shape.vocab, 75)
    sched = [(2, 500)]
    out = model.prefill(torch.from_numpy(ids.astype(np.int32)).to(DEV), sched)
    torch.cuda.synchronize()
    with pytest.raises(B.LazyLLMError) as e:
        B.Generation(model, sched, out, 40)                   # capacity must exceed the prompt
    assert e.value.status == B.LAZYLLM_EINVAL
    with pytest.raises(B.LazyLLMError) as e:
        B.Generation(model, [(1, 500)], out, 48)              # not the prefill's schedule
    assert e.value.status == B.LAZYLLM_EINVAL
    gen = B.Generation(model, sched, out, 41)
    tok = torch.tensor([3], dtype=torch.int32, device=DEV)
    gen.step(tok)
    with pytest.raises(B.LazyLLMError) as e:
        gen.step(tok)                                         # capacity used up
    assert e.value.status == B.LAZYLLM_ENOSPC
    torch.cuda.synchronize()
    gen.close()
    gen = B.Generation(model, sched, out, 44)
    so = gen.step(torch.tensor([shape.vocab + 5], dtype=torch.int32, device=DEV))
    torch.cuda.synchronize()
    assert so.status & B.LAZYLLM_ST_BAD_TOKEN
    gen.close()


def test_steps_are_bit_identical_across_runs(tiny_wide):
    shape, wb, model = tiny_wide
    ids = synth.make_prompt(260, shape.vocab, 76)
    sched = [(1, 700), (3, 400)]
    logits = []
    for _ in range(2):
        out = model.prefill(torch.from_numpy(ids.astype(np.int32)).to(DEV), sched)
        gen = B.Generation(model, sched, out, 270)
        got = []
        for tok in (4, 5, 6):
            so = gen.step(torch.tensor([tok], dtype=torch.int32, device=DEV))
            torch.cuda.synchronize()
            got.append(so.logits.clone())
        logits.append(got)
        gen.close()
    assert all(torch.equal(a, b) for a, b in zip(*logits))


def test_long_sequence_selection_beyond_lds(tiny):
    """More tokens than the selection kernel keeps in LDS (15360): the step's selection must still
    be exactly the top-k of the GPU's own fp32 scores among the tokens selected a layer below, and
    the rows that ran exactly the selected tokens without K,V."""
    shape, wb, model = tiny
    n = 15500
    ids = synth.make_prompt(n, shape.vocab, 78)
    sched = [(2, 500), (3, 300)]
    out = model.prefill(torch.from_numpy(ids.astype(np.int32)).to(DEV), sched)
    gen = B.Generation(model, sched, out, n + 3)
    torch.cuda.synchronize()
    L = shape.n_layers
    for t, tok in enumerate((5, 6)):
        n_tot = n + t + 1
        had = [gen.view()["has_kv"][l].clone().cpu().numpy().astype(bool) for l in range(L)]
        so = gen.step(torch.tensor([tok], dtype=torch.int32, device=DEV))
        torch.cuda.synchronize()
        assert so.status == 0
        counts = O.keep_counts(n_tot, L, sched)
        prev = np.arange(n_tot)
        for l in range(L):
            m = so.selected(l)
            sel = np.arange(n_tot) if m is None else np.nonzero(m.cpu().numpy())[0]
            assert len(sel) == counts[l]
            if l in (2, 3):
                cand = prev[:-1]
                s32 = so.scores(l - 1).cpu().numpy()[cand]
                order = np.argsort(-s32, kind="stable")[: counts[l] - 1]
                assert np.array_equal(sel, np.sort(np.concatenate([cand[order], [n_tot - 1]])))
            assert np.array_equal(so.ran_pos(l).cpu().numpy(), sel[~had[l][sel]])
            s = so.scores(l).double().cpu().numpy()
            assert abs(s.sum() - 1.0) < 2e-4
            prev = sel
    gen.close()
