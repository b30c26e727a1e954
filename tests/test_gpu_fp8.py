"""Parity of the 8-bit (OFP8 E4M3) GEMM variant, through the C ABI, against the CPU checker:
the row quantiser's codes and scales bit for bit, the product within the rounding of its bf16
output plus the accumulation error of the matrix instruction (the checker accumulates in fp64)."""
import math

import numpy as np
import pytest
import torch

from oracle import fp8_oracle as F
from oracle import lazyllm_oracle as O
from paper_2407_14057_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _bf16_dev(x: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16).to(DEV)


def _f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


def _quantize_gpu(x: torch.Tensor, ldq=None):
    rows, K = x.shape
    ldq = K if ldq is None else ldq
    codes = torch.full((rows, ldq), 0xAA, dtype=torch.uint8, device=DEV)
    scale = torch.full((rows,), -1.0, dtype=torch.float32, device=DEV)
    B.lazyllm_op_quantize_fp8(x, rows, K, x.stride(0), codes, ldq, scale)
    torch.cuda.synchronize()
    return codes, scale


@pytest.mark.parametrize("rows,K", [(1, 8), (5, 200), (300, 4096), (37, 11008), (3, 16384), (130, 704)])
def test_quantiser_codes_and_scales_bit_exact(rows, K):
    rng = np.random.default_rng(rows * 31 + K)
    x = rng.normal(0, 1, (rows, K)).astype(np.float32)
    x *= np.exp(rng.normal(0, 3, (rows, 1))).astype(np.float32)        # rows of very different magnitude
    if rows >= 5:
        x[1] = 0.0                                                       # an all-zero row
        x[2, 1:] = 0.0                                                   # one non-zero entry
        x[3, ::2] = -0.0                                                 # negative zeros
        x[4] *= 1e-30                                                    # tiny magnitudes
    xd = _bf16_dev(x)
    codes, scale = _quantize_gpu(xd)
    ref_codes, ref_scale = F.quantize_rows(_f32(xd))
    assert np.array_equal(scale.cpu().numpy().view(np.uint32), ref_scale.view(np.uint32))
    got = codes.cpu().numpy()
    assert np.array_equal(got, ref_codes), "%d codes differ" % int((got != ref_codes).sum())


def test_quantiser_ties_saturation_and_strides():
    # a row whose largest entry is 448 has scale 1: then every halfway point between neighbouring
    # codes (5 significant bits, exact in bf16) is a tie and must go to the even code
    pos = F.e4m3_decode(np.arange(0x7F, dtype=np.uint8))
    halfway = (pos[:-1] + pos[1:]) / 2
    vals = np.concatenate([[448.0], halfway, -halfway, pos, -pos, np.nextafter(halfway.astype(np.float32), 0)])
    K = (len(vals) + 7) // 8 * 8
    x = np.zeros((2, K), dtype=np.float32)
    x[0, :len(vals)] = vals
    x[1, :len(vals)] = vals[::-1] * 0.5
    x[1, 0] = 448.0
    xd = _bf16_dev(x)
    assert np.array_equal(_f32(xd)[0, 1:1 + len(halfway)], halfway.astype(np.float32))   # exact in bf16
    codes, scale = _quantize_gpu(xd)
    ref_codes, ref_scale = F.quantize_rows(_f32(xd))
    assert scale.cpu().tolist() == [1.0, 1.0] and ref_scale.tolist() == [1.0, 1.0]
    assert np.array_equal(codes.cpu().numpy(), ref_codes)
    assert np.array_equal(ref_codes[0, 1:1 + len(halfway)] % 2, np.zeros(len(halfway), dtype=np.uint8))
    # strided input and output; bytes between the rows of the output stay untouched
    rng = np.random.default_rng(2)
    big = _bf16_dev(rng.normal(0, 1, (9, 96)))
    view = big[:, 8:72]                                                  # K = 64, row stride 96
    codes = torch.full((9, 80), 0xAA, dtype=torch.uint8, device=DEV)
    scale = torch.full((9,), -1.0, dtype=torch.float32, device=DEV)
    B.lazyllm_op_quantize_fp8(big.view(-1)[8:], 9, 64, 96, codes, 80, scale)
    torch.cuda.synchronize()
    ref_codes, ref_scale = F.quantize_rows(_f32(view))
    got = codes.cpu().numpy()
    assert np.array_equal(got[:, :64], ref_codes) and np.all(got[:, 64:] == 0xAA)
    assert np.array_equal(scale.cpu().numpy(), ref_scale)


def _codes_dev(rng, shape):
    """Random finite E4M3 codes (no NaN codes)."""
    c = rng.integers(0, 256, size=shape, dtype=np.uint8)
    c[(c & 0x7F) == 0x7F] = 0x38
    return c


@pytest.mark.parametrize("M,N,K", [(1, 256, 128), (37, 256, 384), (300, 768, 1024), (513, 1536, 640),
                                   (256, 512, 4096), (2100, 768, 256), (777, 4096, 1408)])
@pytest.mark.parametrize("epi", [B.EPI_STORE, B.EPI_RESIDUAL, B.EPI_SWIGLU])
def test_gemm_fp8_from_codes(M, N, K, epi):
    rng = np.random.default_rng(M * 7 + N + K + epi)
    # codes of a realistic spread: quantised Gaussians
    ac, sa = F.quantize_rows(rng.normal(0, 1, (M, K)).astype(np.float32))
    wc, sw = F.quantize_rows(rng.normal(0, 1 / math.sqrt(K), (N, K)).astype(np.float32))
    acc = F.gemm_fp8(ac, sa, wc, sw)
    mag = F.gemm_fp8(ac & 0x7F, sa, wc & 0x7F, sw)                       # sum of the terms' magnitudes
    a_d, w_d = torch.from_numpy(ac).to(DEV), torch.from_numpy(wc).to(DEV)
    sa_d, sw_d = torch.from_numpy(sa).to(DEV), torch.from_numpy(sw).to(DEV)
    if epi == B.EPI_SWIGLU:
        blocks = acc.reshape(M, N // 64, 2, 32)
        ref = (O.silu(blocks[:, :, 0, :]) * blocks[:, :, 1, :]).reshape(M, N // 2)
        Cout = torch.full((M, N // 2), 7.0, dtype=torch.bfloat16, device=DEV)
        B.lazyllm_op_gemm_fp8(a_d, sa_d, w_d, sw_d, Cout, None, M, N, K, K, K, N // 2, epi)
    elif epi == B.EPI_RESIDUAL:
        R = _bf16_dev(rng.normal(0, 1, (M, N)))
        ref = _f32(R).astype(np.float64) + acc
        Cout = R.clone()
        B.lazyllm_op_gemm_fp8(a_d, sa_d, w_d, sw_d, Cout, Cout, M, N, K, K, K, N, epi)
    else:
        ref = acc
        Cout = torch.full((M, N), 7.0, dtype=torch.bfloat16, device=DEV)
        B.lazyllm_op_gemm_fp8(a_d, sa_d, w_d, sw_d, Cout, None, M, N, K, K, K, N, epi)
    torch.cuda.synchronize()
    got = _f32(Cout).astype(np.float64)
    # bf16 output: half an ulp (2^-8 relative).  The products are exact, but the matrix instruction
    # adds its 64 products in an internal format and the result to the fp32 accumulator: measured up
    # to 1e-5 of the sum of the terms' magnitudes (it shows where the terms cancel); 3e-5 allowed,
    # still 2^-11 of the 8-bit format's own rounding step.  (Ahead of the SiLU, whose slope is <= 1.1.)
    err = np.abs(got - ref)
    extra = 3e-5 * mag if epi != B.EPI_SWIGLU else 4e-4
    tol = 2.0 ** -8 * np.abs(ref) + extra + 1e-30
    assert not (err > tol).any(), "%d of %d off, worst %.3g" % (int((err > tol).sum()), err.size, float(err.max()))


@pytest.mark.parametrize("M,N,K", [(37, 256, 384), (300, 768, 1024), (2100, 768, 256)])
@pytest.mark.parametrize("epi", [B.EPI_STORE, B.EPI_RESIDUAL, B.EPI_SWIGLU])
def test_gemm_fp8_k_step_major_codes(M, N, K, epi):
    """Weight codes stored K-step-major (the model's form) give the bits of the row-major codes."""
    rng = np.random.default_rng(M + N + K + epi)
    a_d = torch.from_numpy(_codes_dev(rng, (M, K))).to(DEV)
    w_d = torch.from_numpy(_codes_dev(rng, (N, K))).to(DEV)
    sa_d = torch.from_numpy(np.exp(rng.normal(0, 1, M)).astype(np.float32) * 1e-2).to(DEV)
    sw_d = torch.from_numpy(np.exp(rng.normal(0, 1, N)).astype(np.float32) * 1e-2).to(DEV)
    wb = torch.empty_like(w_d)
    B.lazyllm_op_pack_weight_ksteps(w_d, N, K // 2, K // 2, wb)
    torch.cuda.synchronize()
    assert torch.equal(wb.view(K // 128, N, 128), w_d.view(N, K // 128, 128).permute(1, 0, 2).contiguous())
    R = _bf16_dev(rng.normal(0, 1, (M, N)))
    outs = []
    for w, flag in ((w_d, 0), (wb, 1 << 29)):
        if epi == B.EPI_SWIGLU:
            Cout = torch.full((M, N // 2), 7.0, dtype=torch.bfloat16, device=DEV)
            B.lazyllm_op_gemm_fp8(a_d, sa_d, w, sw_d, Cout, None, M, N, K, K, K, N // 2, epi | flag)
        else:
            Cout = R.clone()
            B.lazyllm_op_gemm_fp8(a_d, sa_d, w, sw_d, Cout, Cout if epi == B.EPI_RESIDUAL else None, M, N, K, K, K, N, epi | flag)
        torch.cuda.synchronize()
        outs.append(Cout)
    assert torch.equal(outs[0], outs[1])


def test_gemm_fp8_all_code_pairs_and_scales():
    """Every code against every code (K = 128 holds each A code in one row block), distinct scales
    per row and per column: a swapped operand, a wrong scale index or a wrong format would show."""
    rng = np.random.default_rng(9)
    M, N, K = 256, 256, 128
    ac = np.repeat(np.arange(256, dtype=np.uint8)[:, None], K, axis=1)
    ac[(ac & 0x7F) == 0x7F] = 0
    wc = _codes_dev(rng, (N, K))
    wc[:, 0] = np.arange(256, dtype=np.uint8)
    wc[(wc & 0x7F) == 0x7F] = 0
    sa = np.exp(rng.normal(0, 1, M)).astype(np.float32) * 1e-3
    sw = np.exp(rng.normal(0, 1, N)).astype(np.float32) * 1e-3
    ref = F.gemm_fp8(ac, sa, wc, sw)
    mag = F.gemm_fp8(ac & 0x7F, sa, wc & 0x7F, sw)
    Cout = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
    B.lazyllm_op_gemm_fp8(torch.from_numpy(ac).to(DEV), torch.from_numpy(sa).to(DEV),
                          torch.from_numpy(wc).to(DEV), torch.from_numpy(sw).to(DEV), Cout, None,
                          M, N, K, K, K, N, B.EPI_STORE)
    torch.cuda.synchronize()
    got = _f32(Cout).astype(np.float64)
    # Rows of A that hold only subnormal codes (exponent field 0) lose up to three more bits: the
    # instruction adds its products in a window below the largest exponent FIELD sum, and a
    # subnormal's leading zeros use up part of it (measured 2e-4 of the magnitudes; such rows do not
    # occur after the row quantiser, whose largest entry is always the normal 448).
    sub_row = ((ac[:, 0] >> 3) & 0xF) == 0
    extra = np.where(sub_row, 4e-4, 3e-5)[:, None] * mag
    err = np.abs(got - ref)
    assert np.all(err <= 2.0 ** -8 * np.abs(ref) + extra + 1e-30), int((err > 2.0 ** -8 * np.abs(ref) + extra + 1e-30).sum())


def test_quantise_then_multiply_full_size_sampled():
    """The gate/up projection of the 7B shape at the headline prompt length, from bf16 operands:
    quantiser and product together, checked on sampled rows against the checker, and against the
    exact product within the format's precision."""
    rng = np.random.default_rng(77)
    M, N, K = 3376, 22016, 4096
    A = _bf16_dev(rng.normal(0, 1, (M, K)))
    W = torch.empty((N, K), dtype=torch.bfloat16, device=DEV)
    for r0 in range(0, N, 4096):
        r1 = min(N, r0 + 4096)
        W[r0:r1] = _bf16_dev(rng.normal(0, 1 / math.sqrt(K), (r1 - r0, K)))
    ac, sa = _quantize_gpu(A)
    wc, sw = _quantize_gpu(W)
    Cout = torch.empty((M, N // 2), dtype=torch.bfloat16, device=DEV)
    B.lazyllm_op_gemm_fp8(ac, sa, wc, sw, Cout, None, M, N, K, K, K, N // 2, B.EPI_SWIGLU)
    torch.cuda.synchronize()
    rows = np.array([0, 1, 255, 256, 1777, 3071, 3072, 3375])            # tile edges and the ragged last tile
    blocks = np.concatenate([np.arange(0, 8), np.arange(170, 178), np.arange(336, 344)])   # 64-row blocks of W
    w_rows = (blocks[:, None] * 64 + np.arange(64)[None, :]).reshape(-1)
    out_cols = (blocks[:, None] * 32 + np.arange(32)[None, :]).reshape(-1)
    a_rows, w_sel = _f32(A[rows]), _f32(W[torch.from_numpy(w_rows).to(DEV)])
    rc, rs = F.quantize_rows(a_rows)
    assert np.array_equal(ac[rows].cpu().numpy(), rc) and np.array_equal(sa[rows].cpu().numpy(), rs)
    wq, ws = F.quantize_rows(w_sel)
    assert np.array_equal(sw.cpu().numpy()[w_rows], ws)
    assert np.array_equal(wc.cpu().numpy()[w_rows], wq)
    acc = F.gemm_fp8(rc, rs, wq, ws).reshape(len(rows), len(blocks), 2, 32)
    ref = (O.silu(acc[:, :, 0, :]) * acc[:, :, 1, :]).reshape(len(rows), len(blocks) * 32)
    got = _f32(Cout[rows]).astype(np.float64)[:, out_cols]
    assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 4e-4)
    # against the unquantised product: two operands with 2^-4 relative rounding steps give a few
    # per cent of the product's spread
    eb = (a_rows.astype(np.float64) @ w_sel.astype(np.float64).T).reshape(len(rows), len(blocks), 2, 32)
    exact_out = (O.silu(eb[:, :, 0, :]) * eb[:, :, 1, :]).reshape(len(rows), len(blocks) * 32)
    assert np.sqrt(np.mean((got - exact_out) ** 2)) < 0.06 * np.sqrt(np.mean(exact_out ** 2))


def test_fp8_argument_checks():
    x = torch.zeros((4, 64), dtype=torch.bfloat16, device=DEV)
    codes = torch.zeros((4, 64), dtype=torch.uint8, device=DEV)
    scale = torch.zeros(4, dtype=torch.float32, device=DEV)
    with pytest.raises(B.LazyLLMError):
        B.lazyllm_op_quantize_fp8(x, 4, 60, 64, codes, 64, scale)        # K % 8
    with pytest.raises(B.LazyLLMError):
        B.lazyllm_op_quantize_fp8(x, 4, 64, 32, codes, 64, scale)        # stride below K
    with pytest.raises(B.LazyLLMError):
        B.lazyllm_op_quantize_fp8(x, 4, 16392, 16392, codes, 16392, scale)   # K above the limit
    a = torch.zeros((4, 128), dtype=torch.uint8, device=DEV)
    w = torch.zeros((256, 128), dtype=torch.uint8, device=DEV)
    sw = torch.zeros(256, dtype=torch.float32, device=DEV)
    out = torch.zeros((4, 256), dtype=torch.bfloat16, device=DEV)
    for bad in (dict(N=128), dict(K=64), dict(lda=120), dict(ldc=100), dict(epi=B.EPI_RESIDUAL), dict(epi=3)):
        kw = dict(M=4, N=256, K=128, lda=128, ldw=128, ldc=256, epi=B.EPI_STORE)
        kw.update(bad)
        with pytest.raises(B.LazyLLMError):
            B.lazyllm_op_gemm_fp8(a, scale, w, sw, out, None, kw["M"], kw["N"], kw["K"], kw["lda"],
                                  kw["ldw"], kw["ldc"], kw["epi"])
    B.lazyllm_op_gemm_fp8(a, scale, w, sw, out, None, 0, 256, 128, 128, 128, 256, B.EPI_STORE)   # M = 0: nothing to do


# ------------------------------------------------------------ the prefill with 8-bit projections

from paper_2407_14057_amd import synth
from test_gpu_prefill import check_against_checker, _run, _to_dev

# The checker quantises the same way, so the two differ only where bf16 storage noise moves an
# activation across a rounding boundary of the 8-bit format: a few per cent of the entries, each
# then off by one 8-bit step (2^-4 relative) -- about four times the 16-bit path's noise.
# Measured on the small model: K, V 0.075 of their largest entry, scores 1.4e-2, logits 0.04 of their range.
TOL8 = {"kv": 1e-1, "s64": 4e-2, "s16": 4e-2, "logits": 6e-2, "aux": 0.1, "band": 3e-2}


@pytest.fixture(scope="module")
def tiny8():
    w = synth.make_weights(synth.TINY_FP8, 1001, "cpu", gain_jitter=0.3)
    model = B.Model(synth.TINY_FP8.as_dict(), _to_dev(w), DEV)
    yield synth.TINY_FP8, synth.weights_to_host_bits(w), model
    model.close()


def test_tiny512_fp8_matches_checker(tiny8):
    shape, wb, model = tiny8
    wl = synth.WORKLOADS["tiny512_fp8"]
    inp = synth.make_workload_inputs(wl)
    out = _run(model, inp["token_ids"], wl.schedule)
    assert out.status == 0 and out.n_tokens == [512, 512, 359, 180]
    rep = check_against_checker(shape, wb, inp["token_ids"], list(wl.schedule), out, verbose="tiny512_fp8",
                                gemm8=True, tol=TOL8)
    # and it is the 8-bit arithmetic that ran: the 16-bit checker is further away than the 8-bit one
    ref = O.prefill(shape.as_dict(), wb, inp["token_ids"], [], keep_hidden=False)
    dense = _run(model, inp["token_ids"], [])
    l16 = np.abs(dense.logits[0].cpu().numpy() - ref.logits).max() / (ref.logits.max() - ref.logits.min())
    ref8 = O.prefill(shape.as_dict(), wb, inp["token_ids"], [], gemm8=True)
    l8 = np.abs(dense.logits[0].cpu().numpy() - ref8.logits).max() / (ref8.logits.max() - ref8.logits.min())
    print("dense logits vs 16-bit checker %.4f, vs 8-bit checker %.4f" % (l16, l8))
    assert l8 < l16


@pytest.mark.parametrize("n,sched", [(1, []), (65, [(1, 900), (2, 500), (3, 100)]), (300, [(3, 1)]),
                                     (777, [(1, 300)])])
def test_tiny_fp8_shapes_and_schedules(tiny8, n, sched):
    shape, wb, model = tiny8
    ids = synth.make_prompt(n, shape.vocab, 300 + n)
    out = _run(model, ids, sched)
    assert out.status == 0
    check_against_checker(shape, wb, ids, sched, out, verbose="fp8 n=%d %s" % (n, sched), gemm8=True, tol=TOL8)


def test_fp8_runs_are_bit_identical_and_batches_are_independent(tiny8):
    shape, wb, model = tiny8
    lens = [130, 512, 77]
    ids = np.concatenate([synth.make_prompt(n, shape.vocab, 900 + n) for n in lens])
    cu = [0, 130, 642, 719]
    sched = [(1, 800), (3, 400)]
    a = _run(model, ids, sched, cu=cu)
    snap = a.logits.clone()
    b = _run(model, ids, sched, cu=cu)
    assert torch.equal(snap, b.logits)
    for i, n in enumerate(lens):
        single = _run(model, ids[cu[i]:cu[i + 1]], sched)
        assert torch.equal(single.logits[0], snap[i])


def test_decoding_steps_after_an_8bit_prefill(tiny8):
    """Decoding steps compute in 16-bit arithmetic on every model; after a prefill with 8-bit
    projections they continue from the K,V and Aux Cache that prefill left.  Same comparison as
    for the 16-bit model, the checker's prefill in the 8-bit mode, tolerances of the 8-bit prefill
    where its results are compared (caches), wider bands where they feed the steps."""
    from test_gpu_decode import run_case
    shape, wb, model = tiny8
    ids = synth.make_prompt(300, shape.vocab, 77)
    rep = run_case(shape, wb, model, ids, [(1, 800), (3, 400)], [5, 17, 900, 3], label="decode after fp8 prefill",
                   band=3e-2, s_tol=(3e-2, 3e-2), gemm8=True, logit_tol=3e-2, kv_tol=1e-1, aux_tol=0.1)
    assert sum(sum(r) for r in rep["revived"]) > 0            # revivals happened


@pytest.mark.parametrize("heads,hd,kv", [(4, 64, 2), (2, 128, 1)])
def test_fp8_with_shared_kv_heads_batches_and_flags(heads, hd, kv):
    """The 8-bit projections together with the other variants of the path: grouped-query attention
    (a narrower k/v part of the fused QKV matrix), a ragged batch, hidden-state copies."""
    import dataclasses
    shape = dataclasses.replace(synth.TINY_FP8, n_heads=heads, head_dim=hd, d_model=heads * hd, n_kv_heads=kv)
    w = synth.make_weights(shape, 1200 + heads + kv, "cpu", gain_jitter=0.2)
    model = B.Model(shape.as_dict(), _to_dev(w), DEV)
    wb = synth.weights_to_host_bits(w)
    sched = [(1, 800), (3, 300)]
    lens = [300, 65]
    ids = np.concatenate([synth.make_prompt(n, shape.vocab, 950 + n) for n in lens])
    cu = [0, 300, 365]
    out = _run(model, ids, sched, cu=cu, flags=B.LAZYLLM_KEEP_HIDDEN)
    assert out.status == 0 and out.k(0).shape == (365, kv, hd)
    for b in range(2):
        check_against_checker(shape, wb, ids[cu[b]:cu[b + 1]], sched, out, seq=b,
                              verbose="fp8 gqa H=%d hd=%d kv=%d seq %d" % (heads, hd, kv, b), gemm8=True, tol=TOL8)
    plain = _run(model, ids, sched, cu=cu)
    assert torch.equal(plain.logits, out.logits)
    model.close()
