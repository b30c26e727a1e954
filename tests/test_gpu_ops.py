"""Kernel-level parity: each step of the path, through the C ABI, against the CPU checker on
the same seeded inputs.  Sizes span several tiles plus a ragged tail; integer and index
results must be bit-exact, floating point within the tolerance stated at each test."""
import math

import numpy as np
import pytest
import torch

from oracle import lazyllm_oracle as O
from paper_2407_14057_amd import binding as B
from paper_2407_14057_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _bf16_dev(x: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16).to(DEV)


def _f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def _rand_bf16(rng, shape, std=1.0):
    return _bf16_dev(rng.normal(0.0, std, size=shape))


# bf16 output: half an ulp of the result (2^-9 relative) plus fp32 accumulation noise
def _assert_bf16_close(got: np.ndarray, ref: np.ndarray, scale: float, what: str):
    err = np.abs(got - ref)
    tol = 2.0 ** -8 * np.abs(ref) + 2e-3 * scale
    bad = err > tol
    assert not bad.any(), "%s: %d of %d off, worst %.3g (ref %.3g)" % (
        what, int(bad.sum()), bad.size, float(err.max()), float(np.abs(ref).max()))


# ------------------------------------------------------------------------------------ GEMM

@pytest.mark.parametrize("M,N,K", [(1, 128, 64), (37, 256, 128), (300, 768, 256), (513, 1536, 704),
                                   (130, 4096, 4096), (2100, 768, 256), (2100, 6144, 512)])
@pytest.mark.parametrize("epi", [B.EPI_STORE, B.EPI_RESIDUAL, B.EPI_SWIGLU])
def test_gemm(M, N, K, epi):
    rng = np.random.default_rng(M * 7 + N + K + epi)
    A = _rand_bf16(rng, (M, K))
    W = _rand_bf16(rng, (N, K), 1.0 / math.sqrt(K))
    a, w = _f64(A), _f64(W)
    acc = a @ w.T
    if epi == B.EPI_SWIGLU:
        # library layout: rows 64j..64j+31 gate, 64j+32..64j+63 up
        blocks = acc.reshape(M, N // 64, 2, 32)
        ref = (O.silu(blocks[:, :, 0, :]) * blocks[:, :, 1, :]).reshape(M, N // 2)
        Cout = torch.full((M, N // 2), 7.0, dtype=torch.bfloat16, device=DEV)
        B.lazyllm_op_gemm(A, W, Cout, None, M, N, K, K, K, N // 2, epi)
    elif epi == B.EPI_RESIDUAL:
        R = _rand_bf16(rng, (M, N))
        ref = _f64(R) + acc
        Cout = R.clone()
        B.lazyllm_op_gemm(A, W, Cout, Cout, M, N, K, K, K, N, epi)      # in place on the residual
    else:
        ref = acc
        Cout = torch.full((M, N), 7.0, dtype=torch.bfloat16, device=DEV)
        B.lazyllm_op_gemm(A, W, Cout, None, M, N, K, K, K, N, epi)
    torch.cuda.synchronize()
    _assert_bf16_close(_f64(Cout), ref, 1.0, "gemm")


@pytest.mark.parametrize("M,N,K", [(1, 128, 64), (1, 4096, 4096), (2, 12288, 4096), (7, 4096, 11008), (31, 768, 256),
                                   (32, 22016, 4096), (17, 1536, 704)])
@pytest.mark.parametrize("epi", [B.EPI_STORE, B.EPI_RESIDUAL, B.EPI_SWIGLU])
def test_gemm_skinny(M, N, K, epi):
    """The weight-streaming kernel for a handful of token rows (K split over waves and workgroups,
    partial sums added in a fixed order): values, and bit-identical results from run to run."""
    rng = np.random.default_rng(M * 11 + N + K + epi)
    A = _rand_bf16(rng, (M, K))
    W = _rand_bf16(rng, (N, K), 1.0 / math.sqrt(K))
    acc = _f64(A) @ _f64(W).T
    ws = torch.empty(B.lazyllm_op_gemm_workspace_bytes(), dtype=torch.uint8, device=DEV)
    e = epi | (8 << 8)
    outs = []
    for _ in range(2):
        if epi == B.EPI_SWIGLU:
            blocks = acc.reshape(M, N // 64, 2, 32)
            ref = (O.silu(blocks[:, :, 0, :]) * blocks[:, :, 1, :]).reshape(M, N // 2)
            Cout = torch.full((M, N // 2), 7.0, dtype=torch.bfloat16, device=DEV)
            B.lazyllm_op_gemm(A, W, Cout, None, M, N, K, K, K, N // 2, e, workspace=ws)
        elif epi == B.EPI_RESIDUAL:
            R = _rand_bf16(np.random.default_rng(5), (M, N))
            ref = _f64(R) + acc
            Cout = R.clone()
            B.lazyllm_op_gemm(A, W, Cout, Cout, M, N, K, K, K, N, e, workspace=ws)
        else:
            ref = acc
            Cout = torch.full((M, N), 7.0, dtype=torch.bfloat16, device=DEV)
            B.lazyllm_op_gemm(A, W, Cout, None, M, N, K, K, K, N, e, workspace=ws)
        torch.cuda.synchronize()
        _assert_bf16_close(_f64(Cout), ref, 1.0, "skinny gemm")
        outs.append(Cout.clone())
    assert torch.equal(outs[0], outs[1])


@pytest.mark.parametrize("cfg,M,N,K", [(5, 1100, 22016, 192), (5, 2100, 22016, 64), (5, 1300, 16384, 128),
                                       (7, 1100, 22016, 192), (7, 1000, 16384, 64), (7, 2100, 22016, 256)])
def test_gemm_swiglu_walks_several_tiles_per_workgroup(cfg, M, N, K):
    """More tiles than compute units: with a workspace (its ticket counters) the SiLU*mul form of
    the ping-pong kernel walks them, a workgroup drawing two to four tiles in turn with the next
    tile's first K step copied during the last step of the current one.  Odd and even numbers of K
    steps (the stage that holds step 0 alternates or not), a single K step (no walk: one workgroup
    per tile), a ragged last tile row; every element against the definition, twice in a row (the
    first launch must leave the counters zero), and the same bits without a workspace."""
    rng = np.random.default_rng(cfg * 1000 + M + N + K)
    ws = torch.empty(B.lazyllm_op_gemm_workspace_bytes(), dtype=torch.uint8, device=DEV)
    A = _rand_bf16(rng, (M, K))
    W = _rand_bf16(rng, (N, K), 1.0 / math.sqrt(K))
    acc = _f64(A) @ _f64(W).T
    blocks = acc.reshape(M, N // 64, 2, 32)
    ref = (O.silu(blocks[:, :, 0, :]) * blocks[:, :, 1, :]).reshape(M, N // 2)
    Cout = torch.full((M, N // 2), 7.0, dtype=torch.bfloat16, device=DEV)
    B.lazyllm_op_gemm(A, W, Cout, None, M, N, K, K, K, N // 2, B.EPI_SWIGLU | (cfg << 8), workspace=ws)
    torch.cuda.synchronize()
    _assert_bf16_close(_f64(Cout), ref, 1.0, "gemm swiglu, tile walk")
    assert int(ws[-4096:].view(torch.int32).abs().sum()) == 0        # flags and counters back at zero
    # again; the K-step-major weight; an output whose rows are not 16-byte aligned (direct stores);
    # no workspace (one workgroup per tile)
    Wb = torch.empty_like(W)
    B.lazyllm_op_pack_weight_ksteps(W, N, K, K, Wb)
    outs = []
    for w, flag, kw in ((W, 0, {"workspace": ws}), (Wb, 1 << 29, {"workspace": ws}), (W, 0, {})):
        C2 = torch.full((M, N // 2), 7.0, dtype=torch.bfloat16, device=DEV)
        B.lazyllm_op_gemm(A, w, C2, None, M, N, K, K, K, N // 2, B.EPI_SWIGLU | (cfg << 8) | flag, **kw)
        outs.append(C2)
    wide = torch.full((M, N // 2 + 4), 7.0, dtype=torch.bfloat16, device=DEV)
    B.lazyllm_op_gemm(A, W, wide, None, M, N, K, K, K, N // 2 + 4, B.EPI_SWIGLU | (cfg << 8), workspace=ws)
    torch.cuda.synchronize()
    for C2 in outs:
        assert torch.equal(C2, Cout)
    assert torch.equal(wide[:, :N // 2], Cout)
    assert bool((wide[:, N // 2:] == 7.0).all())
    assert int(ws[-4096:].view(torch.int32).abs().sum()) == 0


@pytest.mark.parametrize("M,N,K", [(1, 256, 64), (229, 768, 256), (700, 1536, 704), (355, 512, 128), (130, 256, 1408)])
@pytest.mark.parametrize("epi", [B.EPI_STORE, B.EPI_RESIDUAL, B.EPI_SWIGLU])
def test_gemm_tile_of_32_row_waves(M, N, K, epi):
    """The 128x128 tile cut into four waves of 32x128, and the 128x256 tile on eight such waves with three
    stages (both forced; the forms the rotary epilogue with 128-wide heads uses below the large-tile
    threshold; K of one, two, four and more steps) give the bits of the 64x64-wave tile."""
    rng = np.random.default_rng(M * 3 + N + K + epi)
    A = _rand_bf16(rng, (M, K)); W = _rand_bf16(rng, (N, K), 1.0 / math.sqrt(K))
    R = _rand_bf16(rng, (M, N))
    outs = []
    for cfg in (2, 3, 13, 14):                     # (14: the 256x256 tile on four waves of 128x128)
        if epi == B.EPI_SWIGLU:
            Cout = torch.full((M, N // 2), 7.0, dtype=torch.bfloat16, device=DEV)
            B.lazyllm_op_gemm(A, W, Cout, None, M, N, K, K, K, N // 2, epi | (cfg << 8))
        else:
            Cout = R.clone()
            B.lazyllm_op_gemm(A, W, Cout, Cout if epi == B.EPI_RESIDUAL else None, M, N, K, K, K, N, epi | (cfg << 8))
        torch.cuda.synchronize()
        outs.append(Cout)
    assert all(torch.equal(outs[0], o) for o in outs[1:])
    acc = _f64(A) @ _f64(W).T
    if epi == B.EPI_SWIGLU:
        blocks = acc.reshape(M, N // 64, 2, 32)
        ref = (O.silu(blocks[:, :, 0, :]) * blocks[:, :, 1, :]).reshape(M, N // 2)
    else:
        ref = acc + (_f64(R) if epi == B.EPI_RESIDUAL else 0.0)
    _assert_bf16_close(_f64(outs[1]), ref, 1.0, "gemm 32x128 waves")


@pytest.mark.parametrize("M,N,K", [(1, 128, 64), (3, 384, 704), (8, 4096, 4096), (20, 256, 1408)])
@pytest.mark.parametrize("epi", [B.EPI_STORE, B.EPI_RESIDUAL, B.EPI_SWIGLU])
def test_gemm_skinny_streamed_weight_layout(M, N, K, epi):
    """The weight rewritten as sequential streams (lazyllm_op_pack_weight_stream) must give the
    bits of the row-major weight: the kernel sees the same LDS slots either way."""
    rng = np.random.default_rng(M * 13 + N + K + epi)
    A = _rand_bf16(rng, (M, K))
    Wbig = _rand_bf16(rng, (N, K + 8), 1.0 / math.sqrt(K))      # a row stride above K
    W = Wbig[:, :K]
    Wp = torch.full((N, K), 7.0, dtype=torch.bfloat16, device=DEV)
    B.lazyllm_op_pack_weight_stream(Wbig, N, K, K + 8, Wp)
    # the packed form is a permutation of the 16-byte chunks
    torch.cuda.synchronize()
    a = np.sort(W.contiguous().view(torch.int16).cpu().numpy().reshape(-1, 8).view(np.int64).ravel())
    b = np.sort(Wp.view(torch.int16).cpu().numpy().reshape(-1, 8).view(np.int64).ravel())
    assert np.array_equal(a.reshape(-1), b.reshape(-1))
    ws = torch.empty(B.lazyllm_op_gemm_workspace_bytes(), dtype=torch.uint8, device=DEV)
    R = _rand_bf16(rng, (M, N))
    outs = []
    for w, ldw, flag in ((Wbig, K + 8, 0), (Wp, K, 1 << 30)):
        e = epi | (8 << 8) | flag
        if epi == B.EPI_SWIGLU:
            Cout = torch.full((M, N // 2), 7.0, dtype=torch.bfloat16, device=DEV)
            B.lazyllm_op_gemm(A, w, Cout, None, M, N, K, K, ldw, N // 2, e, workspace=ws)
        else:
            Cout = R.clone()
            B.lazyllm_op_gemm(A, w, Cout, Cout if epi == B.EPI_RESIDUAL else None, M, N, K, K, ldw, N, e, workspace=ws)
        torch.cuda.synchronize()
        outs.append(Cout)
    assert torch.equal(outs[0], outs[1])
    # a packed weight cannot be read by any other kernel
    with pytest.raises(B.LazyLLMError):
        B.lazyllm_op_gemm(A, Wp, outs[0], None, M, N, K, K, K, outs[0].shape[1], B.EPI_STORE | (2 << 8) | (1 << 30), workspace=ws)


@pytest.mark.parametrize("cfg,M,N,K", [(2, 300, 768, 256), (3, 229, 1536, 704), (4, 130, 512, 192), (5, 513, 1536, 704),
                                       (7, 700, 768, 1408), (6, 355, 4096, 1408), (0, 2100, 6144, 512), (0, 37, 256, 128),
                                       (13, 229, 1536, 704), (13, 77, 512, 128), (13, 300, 768, 64), (13, 640, 1024, 192),
                                       (14, 513, 1536, 704), (14, 300, 768, 64), (14, 1, 256, 128), (14, 700, 2048, 1408)])
@pytest.mark.parametrize("epi", [B.EPI_STORE, B.EPI_RESIDUAL, B.EPI_SWIGLU])
def test_gemm_k_step_major_weight_layout(cfg, M, N, K, epi):
    """The weight stored K-step-major (lazyllm_op_pack_weight_ksteps, the form the model keeps) must
    give the bits of the row-major weight in every tile configuration: only addresses change."""
    if cfg == 6 and epi == B.EPI_SWIGLU:
        pytest.skip("the stream-K schedule has no SiLU*mul epilogue")
    rng = np.random.default_rng(cfg * 101 + M + N + K + epi)
    A = _rand_bf16(rng, (M, K))
    Wbig = _rand_bf16(rng, (N, K + 16), 1.0 / math.sqrt(K))
    Wb = torch.full((N, K), 7.0, dtype=torch.bfloat16, device=DEV)
    B.lazyllm_op_pack_weight_ksteps(Wbig, N, K, K + 16, Wb)
    torch.cuda.synchronize()
    want = Wbig[:, :K].reshape(N, K // 64, 64).permute(1, 0, 2).contiguous()
    assert torch.equal(Wb.view(K // 64, N, 64), want)
    ws = torch.empty(B.lazyllm_op_gemm_workspace_bytes(), dtype=torch.uint8, device=DEV)
    R = _rand_bf16(rng, (M, N))
    outs = []
    for w, ldw, flag in ((Wbig, K + 16, 0), (Wb, K, 1 << 29)):
        e = epi | (cfg << 8) | flag
        if epi == B.EPI_SWIGLU:
            Cout = torch.full((M, N // 2), 7.0, dtype=torch.bfloat16, device=DEV)
            B.lazyllm_op_gemm(A, w, Cout, None, M, N, K, K, ldw, N // 2, e, workspace=ws)
        else:
            Cout = R.clone()
            B.lazyllm_op_gemm(A, w, Cout, Cout if epi == B.EPI_RESIDUAL else None, M, N, K, K, ldw, N, e, workspace=ws)
        torch.cuda.synchronize()
        outs.append(Cout)
    assert torch.equal(outs[0], outs[1])


def test_gemm_skinny_refuses_more_than_32_rows():
    A = torch.zeros(33, 64, dtype=torch.bfloat16, device=DEV)
    W = torch.zeros(128, 64, dtype=torch.bfloat16, device=DEV)
    Cout = torch.zeros(33, 128, dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(B.lazyllm_op_gemm_workspace_bytes(), dtype=torch.uint8, device=DEV)
    with pytest.raises(B.LazyLLMError):
        B.lazyllm_op_gemm(A, W, Cout, None, 33, 128, 64, 64, 64, 128, B.EPI_STORE | (8 << 8), workspace=ws)


@pytest.mark.parametrize("M,N,K", [(1, 128, 64), (355, 4096, 4096), (1182, 4096, 1408), (130, 256, 11008),
                                   (700, 384, 192), (5000, 128, 64)])
@pytest.mark.parametrize("epi", [B.EPI_STORE, B.EPI_RESIDUAL])
def test_gemm_stream_k(M, N, K, epi):
    """The stream-K schedule (forced) must give the data-parallel kernel's result up to the
    order of the fp32 partial sums, and the same bits on every run."""
    rng = np.random.default_rng(M + N + K + epi)
    A = _rand_bf16(rng, (M, K)); W = _rand_bf16(rng, (N, K), 1.0 / math.sqrt(K))
    R = _rand_bf16(rng, (M, N))
    ws = torch.empty(B.lazyllm_op_gemm_workspace_bytes(), dtype=torch.uint8, device=DEV)
    ref = _f64(A) @ _f64(W).T + (_f64(R) if epi == B.EPI_RESIDUAL else 0.0)
    outs = []
    for _ in range(2):
        Cout = R.clone()
        B.lazyllm_op_gemm(A, W, Cout, Cout if epi == B.EPI_RESIDUAL else None, M, N, K, K, K, N,
                          epi | (6 << 8), workspace=ws)
        torch.cuda.synchronize()
        outs.append(Cout)
    _assert_bf16_close(_f64(outs[0]), ref, 1.0, "gemm stream-K")
    assert torch.equal(outs[0], outs[1])


@pytest.mark.parametrize("epi,M,N,K", [(B.EPI_SWIGLU, 355, 22016, 256), (B.EPI_SWIGLU, 450, 22016, 128),
                                       (B.EPI_SWIGLU, 600, 22016, 192), (B.EPI_SWIGLU, 1000, 22016, 128),
                                       (B.EPI_RESIDUAL, 600, 4096, 512), (B.EPI_RESIDUAL, 861, 4096, 512),
                                       (B.EPI_RESIDUAL, 861, 4096, 8192), (B.EPI_STORE, 700, 12288, 256)])
def test_gemm_library_choice_with_a_workspace(epi, M, N, K):
    """With a workspace the library may choose the persistent stream-K schedule on its own: gate/up
    with a last round two thirds empty (172 or 344 tiles of either height), the O and down
    projections at 64 - 127 aligned tiles, a last round 0.4 or more empty.  Every element against the
    definition, the same bits twice, flags back at zero."""
    rng = np.random.default_rng(epi * 977 + M + N + K)
    A = _rand_bf16(rng, (M, K))
    W = _rand_bf16(rng, (N, K), 1.0 / math.sqrt(K))
    acc = _f64(A) @ _f64(W).T
    ws = torch.empty(B.lazyllm_op_gemm_workspace_bytes(), dtype=torch.uint8, device=DEV)
    outs = []
    for _ in range(2):
        if epi == B.EPI_SWIGLU:
            blocks = acc.reshape(M, N // 64, 2, 32)
            ref = (O.silu(blocks[:, :, 0, :]) * blocks[:, :, 1, :]).reshape(M, N // 2)
            Cout = torch.full((M, N // 2), 7.0, dtype=torch.bfloat16, device=DEV)
            B.lazyllm_op_gemm(A, W, Cout, None, M, N, K, K, K, N // 2, epi, workspace=ws)
        else:
            if not outs:
                R = _rand_bf16(rng, (M, N))
            ref = acc + (_f64(R) if epi == B.EPI_RESIDUAL else 0.0)
            Cout = R.clone()
            B.lazyllm_op_gemm(A, W, Cout, Cout if epi == B.EPI_RESIDUAL else None, M, N, K, K, K, N, epi,
                              workspace=ws)
        torch.cuda.synchronize()
        assert int(ws[-4096:].view(torch.int32).abs().sum()) == 0
        outs.append(Cout)
    _assert_bf16_close(_f64(outs[0]), ref, 1.0, "gemm, library's choice")
    assert torch.equal(outs[0], outs[1])


@pytest.mark.parametrize("cfg", [9, 10])
@pytest.mark.parametrize("M,N,K", [(1, 256, 64), (300, 768, 256), (2364, 4096, 1024), (1182, 4096, 4096),
                                   (3376, 2048, 512), (700, 22016, 256), (5000, 256, 128), (8192, 8192, 128),
                                   (600, 4096, 512), (1000, 4096, 704), (1536, 4096, 256)])
@pytest.mark.parametrize("epi", [B.EPI_STORE, B.EPI_RESIDUAL, B.EPI_SWIGLU])
def test_gemm_persistent_stream_k(cfg, M, N, K, epi):
    """The persistent stream-K schedule of the ping-pong tiles (forced): shapes with fewer tiles than
    CUs (every tile cut into several K pieces; 48, 64, 80 and 96 tiles of 256 rows take a grid of five,
    four, three and two workgroups per tile), with whole data-parallel rounds plus a cut remainder,
    with exactly whole rounds, and a single K step.  Same result as the plain product up to the order
    of the fp32 partial sums, the same bits on every run, flags left at zero, no wait given up."""
    rng = np.random.default_rng(M + N + K + epi + cfg)
    A = _rand_bf16(rng, (M, K)); W = _rand_bf16(rng, (N, K), 1.0 / math.sqrt(K))
    ws = torch.empty(B.lazyllm_op_gemm_workspace_bytes(), dtype=torch.uint8, device=DEV)
    acc = _f64(A) @ _f64(W).T
    if epi == B.EPI_SWIGLU:
        blocks = acc.reshape(M, N // 64, 2, 32)
        ref = (O.silu(blocks[:, :, 0, :]) * blocks[:, :, 1, :]).reshape(M, N // 2)
        R = None
    else:
        R = _rand_bf16(rng, (M, N))
        ref = acc + (_f64(R) if epi == B.EPI_RESIDUAL else 0.0)
    outs = []
    for _ in range(2):
        if epi == B.EPI_SWIGLU:
            Cout = torch.full((M, N // 2), 7.0, dtype=torch.bfloat16, device=DEV)
            B.lazyllm_op_gemm(A, W, Cout, None, M, N, K, K, K, N // 2, epi | (cfg << 8), workspace=ws)
        else:
            Cout = R.clone()
            B.lazyllm_op_gemm(A, W, Cout, Cout if epi == B.EPI_RESIDUAL else None, M, N, K, K, K, N,
                              epi | (cfg << 8), workspace=ws)
        torch.cuda.synchronize()
        outs.append(Cout)
        tail = ws[-4096:].view(torch.int32)
        assert int(tail.abs().sum().item()) == 0          # flags consumed and reset, no wait given up
    _assert_bf16_close(_f64(outs[0]), ref, 1.0, "gemm persistent stream-K")
    assert torch.equal(outs[0], outs[1])


def _ssq_fixed(rows_f64):
    """Row sums of squares in the library's 2^-32 fixed point (from fp64, for inputs)."""
    return torch.from_numpy(np.floor((rows_f64 ** 2).sum(axis=1) * 2.0 ** 32).astype(np.uint64).view(np.int64)).to(DEV)


@pytest.mark.parametrize("M,N,K", [(1, 128, 64), (37, 256, 128), (513, 1536, 704), (355, 4096, 4096),
                                   (2100, 6144, 512)])
@pytest.mark.parametrize("epi", [B.EPI_STORE, B.EPI_SWIGLU])
def test_gemm_with_rmsnorm_folded_in(M, N, K, epi):
    """C = rmsnorm(A) W^T with the 1/rms factor applied to the product's rows (gain 1)."""
    rng = np.random.default_rng(M + 3 * N + K + epi)
    A = _rand_bf16(rng, (M, K), 0.7)
    W = _rand_bf16(rng, (N, K), 1.0 / math.sqrt(K))
    a, w = _f64(A), _f64(W)
    eps = 1e-5
    acc = O.rmsnorm(a, np.ones(K), eps) @ w.T
    ssq = _ssq_fixed(a)
    cleared = torch.full((M + 2,), 77, dtype=torch.int64, device=DEV)
    if epi == B.EPI_SWIGLU:
        blocks = acc.reshape(M, N // 64, 2, 32)
        ref = (O.silu(blocks[:, :, 0, :]) * blocks[:, :, 1, :]).reshape(M, N // 2)
        Cout = torch.full((M, N // 2), 7.0, dtype=torch.bfloat16, device=DEV)
        B.lazyllm_op_gemm_rmsnorm(A, W, Cout, None, M, N, K, K, K, N // 2, epi, ssq_in=ssq, eps=eps,
                                  ssq_clear=cleared)
    else:
        ref = acc
        Cout = torch.full((M, N), 7.0, dtype=torch.bfloat16, device=DEV)
        B.lazyllm_op_gemm_rmsnorm(A, W, Cout, None, M, N, K, K, K, N, epi, ssq_in=ssq, eps=eps,
                                  ssq_clear=cleared)
    torch.cuda.synchronize()
    _assert_bf16_close(_f64(Cout), ref, 1.0, "gemm+rmsnorm")
    c = cleared.cpu().numpy()
    assert np.all(c[:M] == 0) and np.all(c[M:] == 77)      # exactly rows 0..M-1 are zeroed


@pytest.mark.parametrize("cfg,M,N,K", [(5, 1100, 22016, 192), (5, 2100, 22016, 128), (7, 1000, 22016, 192),
                                       (0, 1182, 22016, 256), (0, 355, 22016, 128)])
def test_gemm_swiglu_tile_walk_with_rmsnorm_folded_in(cfg, M, N, K):
    """The SiLU*mul GEMM in the form the prefill launches it -- RMSNorm's row scale folded into the
    epilogue, a workspace, more tiles than compute units -- where a workgroup fetches the row
    scales of its NEXT tile during the last K step of the current one (and, at 355 rows, under the
    persistent stream-K schedule).  Every element against the definition, same bits twice."""
    rng = np.random.default_rng(cfg * 31 + M + N + K)
    A = _rand_bf16(rng, (M, K), 0.7)
    A[: M // 2] *= 3.0                                    # row scales that differ from tile to tile
    W = _rand_bf16(rng, (N, K), 1.0 / math.sqrt(K))
    a, w = _f64(A), _f64(W)
    eps = 1e-5
    acc = O.rmsnorm(a, np.ones(K), eps) @ w.T
    blocks = acc.reshape(M, N // 64, 2, 32)
    ref = (O.silu(blocks[:, :, 0, :]) * blocks[:, :, 1, :]).reshape(M, N // 2)
    ssq = _ssq_fixed(a)
    ws = torch.empty(B.lazyllm_op_gemm_workspace_bytes(), dtype=torch.uint8, device=DEV)
    outs = []
    for _ in range(2):
        Cout = torch.full((M, N // 2), 7.0, dtype=torch.bfloat16, device=DEV)
        B.lazyllm_op_gemm_rmsnorm(A, W, Cout, None, M, N, K, K, K, N // 2, B.EPI_SWIGLU | (cfg << 8),
                                  ssq_in=ssq, eps=eps, workspace=ws)
        torch.cuda.synchronize()
        assert int(ws[-4096:].view(torch.int32).abs().sum()) == 0
        outs.append(Cout)
    _assert_bf16_close(_f64(outs[0]), ref, 1.0, "gemm+rmsnorm, tile walk")
    assert torch.equal(outs[0], outs[1])


@pytest.mark.parametrize("M,N,K", [(1, 128, 64), (37, 256, 128), (355, 4096, 4096), (1182, 4096, 1408),
                                   (2364, 4096, 512), (3376, 4096, 256)])
def test_gemm_residual_leaves_row_sums_of_squares(M, N, K):
    """The residual epilogue adds each written row's sum of squares (of the bf16 values it
    stored) to ssq_out; integer atomics, so the total is the same on every run."""
    rng = np.random.default_rng(M + N + K)
    A = _rand_bf16(rng, (M, K)); W = _rand_bf16(rng, (N, K), 1.0 / math.sqrt(K))
    R = _rand_bf16(rng, (M, N))
    ws = torch.empty(B.lazyllm_op_gemm_workspace_bytes(), dtype=torch.uint8, device=DEV)
    got = []
    for _ in range(2):
        Cout = R.clone()
        ssq = torch.zeros(M, dtype=torch.int64, device=DEV)
        B.lazyllm_op_gemm_rmsnorm(A, W, Cout, Cout, M, N, K, K, K, N, B.EPI_RESIDUAL, ssq_out=ssq,
                                  workspace=ws)
        torch.cuda.synchronize()
        got.append((Cout, ssq.cpu().numpy().view(np.uint64).astype(np.float64) / 2.0 ** 32))
    ref = (_f64(got[0][0]) ** 2).sum(axis=1)                 # of the values actually stored
    assert np.allclose(got[0][1], ref, rtol=2e-6, atol=1e-6), np.abs(got[0][1] / ref - 1).max()
    assert np.array_equal(got[0][1], got[1][1]) and torch.equal(got[0][0], got[1][0])
    _assert_bf16_close(_f64(got[0][0]), _f64(R) + _f64(A) @ _f64(W).T, 1.0, "gemm residual")


def test_gemm_strided_and_edge_rows_untouched():
    rng = np.random.default_rng(5)
    M, N, K = 70, 256, 128
    lda, ldw, ldc = K + 64, K + 8, N + 128
    A = _rand_bf16(rng, (M, lda)); W = _rand_bf16(rng, (N, ldw), 0.1)
    Cout = torch.full((M + 3, ldc), 7.0, dtype=torch.bfloat16, device=DEV)
    B.lazyllm_op_gemm(A, W, Cout, None, M, N, K, lda, ldw, ldc, B.EPI_STORE)
    torch.cuda.synchronize()
    ref = _f64(A)[:, :K] @ _f64(W)[:, :K].T
    got = _f64(Cout)
    _assert_bf16_close(got[:M, :N], ref, 1.0, "gemm strided")
    assert np.all(got[M:, :] == 7.0) and np.all(got[:, N:] == 7.0)     # nothing written outside


def test_gemm_full_size_sampled():
    """The headline shape's first stage (M=3376, QKV projection), checked on sampled outputs."""
    rng = np.random.default_rng(6)
    M, N, K = 3376, 12288, 4096
    A = torch.randn(M, K, device=DEV, dtype=torch.float32, generator=torch.Generator(DEV).manual_seed(1)).to(torch.bfloat16)
    W = (torch.randn(N, K, device=DEV, dtype=torch.float32, generator=torch.Generator(DEV).manual_seed(2)) * 0.02).to(torch.bfloat16)
    Cout = torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
    B.lazyllm_op_gemm(A, W, Cout, None, M, N, K, K, K, N, B.EPI_STORE)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, 255, 256, M - 1, M - 2], rng.integers(0, M, 40)]))
    cols = np.unique(np.concatenate([[0, 127, 128, 255, 256, N - 1], rng.integers(0, N, 200)]))
    a = _f64(A[torch.from_numpy(rows).to(DEV)])
    w = _f64(W[torch.from_numpy(cols).to(DEV)])
    ref = a @ w.T
    got = _f64(Cout[torch.from_numpy(rows).to(DEV)][:, torch.from_numpy(cols).to(DEV)])
    _assert_bf16_close(got, ref, 1.3, "gemm 7B")


# ------------------------------------------------------------------------------------ RMSNorm

@pytest.mark.parametrize("rows,d", [(1, 256), (5, 256), (131, 4096), (33, 1024)])
def test_rmsnorm(rows, d):
    rng = np.random.default_rng(rows + d)
    h = _rand_bf16(rng, (rows, d), 2.0)
    g = _bf16_dev(1.0 + 0.3 * rng.uniform(-1, 1, d))
    x = torch.empty_like(h)
    B.lazyllm_op_rmsnorm(h, g, x, rows, d, 1e-5)
    torch.cuda.synchronize()
    ref = O.rmsnorm(_f64(h), _f64(g), 1e-5)
    _assert_bf16_close(_f64(x), ref, 1e-3, "rmsnorm")


# ------------------------------------------------------------------------------------ QKV + RoPE, V^T

@pytest.mark.parametrize("rows,H,hd", [(1, 4, 64), (130, 4, 64), (200, 2, 128), (300, 32, 128), (2100, 8, 128)])
def test_qkv_rope(rows, H, hd):
    rng = np.random.default_rng(rows + H + hd)
    d = H * hd
    x = _rand_bf16(rng, (rows, d))
    w = _rand_bf16(rng, (3 * d, d), 1.0 / math.sqrt(d))
    pos_np = np.sort(rng.choice(9000, size=rows, replace=False)).astype(np.int32)
    pos = torch.from_numpy(pos_np).to(DEV)
    max_pos = int(pos_np.max())
    table = torch.empty((max_pos + 1) * (hd // 2) * 2, dtype=torch.float32, device=DEV)
    q = torch.full((rows, d), 3.0, dtype=torch.bfloat16, device=DEV)
    k = torch.full_like(q, 3.0); v = torch.full_like(q, 3.0)
    B.lazyllm_op_qkv_rope(x, w, pos, max_pos, table, q, k, v, rows, H, hd, 10000.0)
    torch.cuda.synchronize()
    acc = _f64(x) @ _f64(w).T
    q_ref = O.rope(acc[:, :d].reshape(rows, H, hd), pos_np, 10000.0).reshape(rows, d)
    k_ref = O.rope(acc[:, d:2 * d].reshape(rows, H, hd), pos_np, 10000.0).reshape(rows, d)
    _assert_bf16_close(_f64(q), q_ref, 1.0, "q")
    _assert_bf16_close(_f64(k), k_ref, 1.0, "k")
    _assert_bf16_close(_f64(v), acc[:, 2 * d:], 1.0, "v")
    # one rounding only: almost every element is THE nearest bf16 of the fp64 result
    exact = (_f64(q) == O.round_to_bf16(q_ref)).mean()
    assert exact > 0.99, exact


@pytest.mark.parametrize("rows,H,hd", [(1, 4, 64), (130, 4, 64), (200, 2, 128), (64, 32, 128)])
def test_v_transpose(rows, H, hd):
    rng = np.random.default_rng(rows + H + hd + 1)
    d = H * hd
    v = _rand_bf16(rng, (rows, d))
    vt_ld = (rows + 63) // 64 * 64 + 64
    vt = torch.full((d, vt_ld), 5.0, dtype=torch.bfloat16, device=DEV)
    B.lazyllm_op_v_transpose(v, vt, vt_ld, rows, H, hd)
    torch.cuda.synchronize()
    vtn = _f64(vt)
    assert np.array_equal(vtn[:, :rows], _f64(v).T)                        # transposed copy
    pad = (rows + 63) // 64 * 64
    assert np.all(vtn[:, rows:pad] == 0.0)                                 # tail of the last tile zeroed
    assert np.all(vtn[:, pad:] == 5.0)                                     # nothing beyond


# ------------------------------------------------------------------------------------ attention

def _attention_case(rows, H, hd, seed):
    rng = np.random.default_rng(seed)
    d = H * hd
    q = _rand_bf16(rng, (rows, d)); k = _rand_bf16(rng, (rows, d)); v = _rand_bf16(rng, (rows, d))
    pad = (rows + 63) // 64 * 64
    vt = torch.zeros(d, pad, dtype=torch.bfloat16, device=DEV)
    vt[:, :rows] = v.t()
    o = torch.full((rows, d), 9.0, dtype=torch.bfloat16, device=DEV)
    B.lazyllm_op_attention(q, k, vt.contiguous(), pad, o, rows, H, hd)
    torch.cuda.synchronize()
    sh = (rows, H, hd)
    o_ref, _ = O.causal_attention(_f64(q).reshape(sh), _f64(k).reshape(sh), _f64(v).reshape(sh))
    return _f64(o), o_ref.reshape(rows, d)


@pytest.mark.parametrize("rows", [1, 2, 31, 63, 64, 65, 127, 128, 129, 200, 515])
@pytest.mark.parametrize("H,hd", [(4, 64), (2, 128)])
def test_attention(rows, H, hd):
    got, ref = _attention_case(rows, H, hd, rows * 3 + hd)
    # probabilities are rounded to bf16 before the second product: 2^-9 relative per term
    err = np.abs(got - ref)
    assert err.max() < 2e-2, "worst %.3g" % err.max()
    assert np.sqrt((err ** 2).mean()) < 3e-3


def test_attention_sharp_rows():
    """Large logits: the running-max rescale must not lose the dominant key."""
    rows, H, hd = 300, 2, 128
    rng = np.random.default_rng(77)
    d = H * hd
    q = _rand_bf16(rng, (rows, d), 4.0); k = _rand_bf16(rng, (rows, d), 4.0); v = _rand_bf16(rng, (rows, d))
    pad = (rows + 63) // 64 * 64
    vt = torch.zeros(d, pad, dtype=torch.bfloat16, device=DEV); vt[:, :rows] = v.t()
    o = torch.empty(rows, d, dtype=torch.bfloat16, device=DEV)
    B.lazyllm_op_attention(q, k, vt.contiguous(), pad, o, rows, H, hd)
    torch.cuda.synchronize()
    sh = (rows, H, hd)
    o_ref, _ = O.causal_attention(_f64(q).reshape(sh), _f64(k).reshape(sh), _f64(v).reshape(sh))
    assert np.abs(_f64(o) - o_ref.reshape(rows, d)).max() < 3e-2


@pytest.mark.parametrize("rows,H,hd", [(2049, 32, 128), (2364, 32, 128), (3376, 32, 128), (1100, 64, 64), (1281, 64, 64)])
def test_attention_headline_form(rows, H, hd):
    """The kernel form the 7B workloads launch (more than 256 query blocks of 256 rows over all heads:
    8 waves per workgroup in two half-step groups, 4 stages, fragment ring), with 128-wide heads and
    with 64-wide ones (a ring of 8 fragments), element by element against the checker's full
    attention maps."""
    got, ref = _attention_case(rows, H, hd, rows + 11)
    err = np.abs(got - ref)
    assert err.max() < 2e-2, "worst %.3g" % err.max()
    assert np.sqrt((err ** 2).mean()) < 3e-3
    # rows past the first 256-query block see several key steps: no row is left at its fill value
    assert np.abs(got).max() < 8.0


def test_attention_headline_form_sharp_rows():
    """Large, uneven logits at the headline shape: late keys that exceed the running maximum by
    far more than the lazy-rescale threshold, so the accumulator rescale path runs in the 8-wave
    form too."""
    rows, H, hd = 2100, 32, 128
    rng = np.random.default_rng(78)
    d = H * hd
    q = _rand_bf16(rng, (rows, d), 3.0); k = _rand_bf16(rng, (rows, d), 3.0); v = _rand_bf16(rng, (rows, d))
    # every 97th key is much larger: whoever sees it first must raise its reference point
    k[::97] *= 3.0
    pad = (rows + 63) // 64 * 64
    vt = torch.zeros(d, pad, dtype=torch.bfloat16, device=DEV); vt[:, :rows] = v.t()
    o = torch.empty(rows, d, dtype=torch.bfloat16, device=DEV)
    B.lazyllm_op_attention(q, k, vt.contiguous(), pad, o, rows, H, hd)
    torch.cuda.synchronize()
    sh = (rows, H, hd)
    o_ref, _ = O.causal_attention(_f64(q).reshape(sh), _f64(k).reshape(sh), _f64(v).reshape(sh))
    assert np.abs(_f64(o) - o_ref.reshape(rows, d)).max() < 3e-2


@pytest.mark.parametrize("rows", [1, 2, 31, 32, 33, 64, 65, 127, 128, 129, 255, 257, 515, 1000, 2364])
@pytest.mark.parametrize("H,hd", [(4, 64), (2, 128), (32, 128)])
def test_attention_score(rows, H, hd):
    """Attention that also leaves Eq. 1's scores (the form the prefill runs)."""
    if rows > 600 and H < 32:
        pytest.skip("long case only at the 7B head count")
    rng = np.random.default_rng(rows * 5 + H)
    d = H * hd
    q = _rand_bf16(rng, (rows, d), 1.5); k = _rand_bf16(rng, (rows, d)); v = _rand_bf16(rng, (rows, d))
    pad = (rows + 63) // 64 * 64
    vt = torch.zeros(d, pad, dtype=torch.bfloat16, device=DEV); vt[:, :rows] = v.t()
    o = torch.full((rows, d), 9.0, dtype=torch.bfloat16, device=DEV)
    o_plain = torch.full((rows, d), 9.0, dtype=torch.bfloat16, device=DEV)
    s = torch.full((rows,), -1.0, dtype=torch.float32, device=DEV)
    scratch = torch.empty(B.lazyllm_op_score_scratch_bytes(rows, H), dtype=torch.uint8, device=DEV)
    B.lazyllm_op_attention_score(q, k, vt.contiguous(), pad, o, s, scratch, rows, H, hd)
    B.lazyllm_op_attention(q, k, vt.contiguous(), pad, o_plain, rows, H, hd)
    torch.cuda.synchronize()
    assert torch.equal(o, o_plain)                       # scoring does not disturb the output
    ref = O.last_row_scores(_f64(q[rows - 1]).reshape(H, hd), _f64(k).reshape(rows, H, hd))
    got = s.cpu().numpy().astype(np.float64)
    assert np.allclose(got, ref, rtol=2e-5, atol=1e-9), np.abs(got / ref - 1).max()
    assert abs(got.sum() - 1.0) < 1e-5
    # same scores as the stand-alone scoring kernels, to fp32 rounding
    s2 = torch.empty(rows, dtype=torch.float32, device=DEV)
    B.lazyllm_op_score(q[rows - 1].contiguous(), k, s2, scratch, rows, H, hd)
    torch.cuda.synchronize()
    assert np.allclose(got, s2.cpu().numpy().astype(np.float64), rtol=2e-5, atol=1e-9)


# ------------------------------------------------------------------------------------ Eq. 1 scoring

@pytest.mark.parametrize("rows", [1, 2, 15, 16, 17, 255, 256, 257, 1000, 3376])
@pytest.mark.parametrize("H,hd", [(4, 64), (32, 128)])
def test_score(rows, H, hd):
    rng = np.random.default_rng(rows + H)
    d = H * hd
    k = _rand_bf16(rng, (rows, d))
    q_last = _rand_bf16(rng, (d,), 1.5)
    s = torch.full((rows,), -1.0, dtype=torch.float32, device=DEV)
    scratch = torch.empty(B.lazyllm_op_score_scratch_bytes(rows, H), dtype=torch.uint8, device=DEV)
    B.lazyllm_op_score(q_last, k, s, scratch, rows, H, hd)
    torch.cuda.synchronize()
    ref = O.last_row_scores(_f64(q_last).reshape(H, hd), _f64(k).reshape(rows, H, hd))
    got = s.cpu().numpy().astype(np.float64)
    # fp32 dot products of exact bf16 products, fast exp: a few 1e-6 relative
    assert np.allclose(got, ref, rtol=2e-5, atol=1e-9), np.abs(got / ref - 1).max()
    assert abs(got.sum() - 1.0) < 1e-5


def test_score_is_deterministic():
    rng = np.random.default_rng(9)
    rows, H, hd = 3376, 32, 128
    k = _rand_bf16(rng, (rows, H * hd)); q_last = _rand_bf16(rng, (H * hd,))
    scratch = torch.empty(B.lazyllm_op_score_scratch_bytes(rows, H), dtype=torch.uint8, device=DEV)
    outs = []
    for _ in range(3):
        s = torch.empty(rows, dtype=torch.float32, device=DEV)
        B.lazyllm_op_score(q_last, k, s, scratch, rows, H, hd)
        torch.cuda.synchronize()
        outs.append(s.cpu().numpy().copy())
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


# ------------------------------------------------------------------------------------ selection

def _select(scores: np.ndarray, k: int):
    m = scores.shape[0]
    s = torch.from_numpy(scores).to(DEV)
    keep = torch.full((k,), -1, dtype=torch.int32, device=DEV)
    prune = torch.full((max(m - k, 1),), -1, dtype=torch.int32, device=DEV)
    B.lazyllm_op_select(s, m, k, keep, prune)
    torch.cuda.synchronize()
    return keep.cpu().numpy(), prune.cpu().numpy()[: m - k]


@pytest.mark.parametrize("kind", synth.SCORE_KINDS)
@pytest.mark.parametrize("m", [1, 2, 63, 64, 65, 1024, 1025, 3376, 8192])
def test_select_bit_exact(kind, m):
    s = synth.make_scores(kind, m, 1000 + m)
    ks = sorted(k for k in {1, 2, max(1, m // 2), max(1, (m * 7 + 9) // 10), max(1, m - 1), m} if k <= m)
    for k in ks:
        keep, prune = _select(s, k)
        rk, rp = O.select_tokens(s, k)
        assert np.array_equal(keep, rk), (kind, m, k)
        assert np.array_equal(prune, rp), (kind, m, k)


def test_select_long_sequence_uses_global_memory_path():
    m = 40000                                      # beyond what the kernel keeps in LDS
    for kind in ("softmax_like", "few_values", "lognormal3"):
        s = synth.make_scores(kind, m, 4242)
        for k in (1, 12000, 39999):
            keep, prune = _select(s, k)
            rk, rp = O.select_tokens(s, k)
            assert np.array_equal(keep, rk) and np.array_equal(prune, rp)


def test_select_last_token_forced_and_negative_scores():
    s = np.linspace(1.0, 0.0, 50, dtype=np.float32)     # the last token has the lowest score
    keep, _ = _select(s, 5)
    assert list(keep) == [0, 1, 2, 3, 49]
    s2 = np.array([-1.0, 3.0, -0.5, 2.0, -7.0], np.float32)
    keep, prune = _select(s2, 3)
    assert list(keep) == [1, 3, 4] and list(prune) == [0, 2]


# ------------------------------------------------------------------------------------ gather

@pytest.mark.parametrize("m,k,d", [(1, 1, 256), (50, 20, 256), (515, 360, 4096), (300, 300, 1024)])
def test_gather_bit_exact(m, k, d):
    rng = np.random.default_rng(m + k)
    h = _rand_bf16(rng, (m, d))
    pos_np = np.sort(rng.choice(10000, size=m, replace=False)).astype(np.int32)
    perm = rng.permutation(m)
    keep_np = np.sort(perm[:k]).astype(np.int32); prune_np = np.sort(perm[k:]).astype(np.int32)
    pos = torch.from_numpy(pos_np).to(DEV)
    keep = torch.from_numpy(keep_np).to(DEV)
    prune = torch.from_numpy(prune_np).to(DEV) if m > k else torch.zeros(1, dtype=torch.int32, device=DEV)
    h_out = torch.empty(k, d, dtype=torch.bfloat16, device=DEV)
    pos_out = torch.empty(k, dtype=torch.int32, device=DEV)
    aux_h = torch.empty(max(m - k, 1), d, dtype=torch.bfloat16, device=DEV)
    aux_pos = torch.empty(max(m - k, 1), dtype=torch.int32, device=DEV)
    B.lazyllm_op_gather(h, pos, keep, k, prune, m - k, h_out, pos_out, aux_h, aux_pos, d)
    torch.cuda.synchronize()
    hb = h.view(torch.int16).cpu().numpy()
    assert np.array_equal(h_out.view(torch.int16).cpu().numpy(), hb[keep_np])
    assert np.array_equal(pos_out.cpu().numpy(), pos_np[keep_np])
    if m > k:
        assert np.array_equal(aux_h.view(torch.int16).cpu().numpy()[: m - k], hb[prune_np])
        assert np.array_equal(aux_pos.cpu().numpy()[: m - k], pos_np[prune_np])


# ------------------------------------------------------------------------------------ LM head

# (rows of 32, 192 and 130 16-byte chunks: a wave's two-chunk step with idle lanes, with a tail, with
#  both; vocabularies that are no multiple of the 4 rows a wave takes at a time or the 64 of a
#  workgroup; a row wider than the fused form takes, which goes through the two-launch form)
@pytest.mark.parametrize("d,V", [(256, 1024), (4096, 32000), (256, 1001), (1536, 1003), (1040, 67), (8, 5),
                                 (40960, 130)])
def test_lm_head(d, V):
    rng = np.random.default_rng(d + V)
    h = _rand_bf16(rng, (d,), 1.5)
    g = _bf16_dev(1.0 + 0.2 * rng.uniform(-1, 1, d))
    w = _rand_bf16(rng, (V, d), 0.02)
    xf = torch.empty(d, dtype=torch.float32, device=DEV)
    logits = torch.empty(V, dtype=torch.float32, device=DEV)
    B.lazyllm_op_lm_head(h, g, w, xf, logits, d, V, 1e-5)
    torch.cuda.synchronize()
    ref = _f64(w) @ O.rmsnorm(_f64(h), _f64(g), 1e-5)
    assert np.allclose(logits.cpu().numpy(), ref, rtol=1e-4, atol=1e-4)
