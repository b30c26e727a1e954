"""The allocation-free Eq. 1 entry point (lazyllm_op_score_static): same results as
lazyllm_op_score, bit for bit, on two calls in a row, the second with a smaller input; the CPU
checker's Eq. 1 bounds both; sizes beyond the static scratch are refused."""
import gc

import numpy as np
import pytest
import torch

from oracle import lazyllm_oracle as O
from paper_2407_14057_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _rand_bf16(rng, shape, scale=1.0):
    return torch.from_numpy((rng.standard_normal(shape) * scale).astype(np.float32)).to(torch.bfloat16).to(DEV)


def _f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def test_static_scratch_scoring_matches_the_buffer_form_on_two_calls_in_a_row():
    rng = np.random.default_rng(77)
    H, hd = 32, 128
    for call, rows in enumerate((3376, 1182)):     # the second call is smaller than the first
        k = _rand_bf16(rng, (rows, H * hd))
        q_last = _rand_bf16(rng, (H * hd,), 1.5)
        s_ref = torch.full((rows,), -1.0, dtype=torch.float32, device=DEV)
        scratch = torch.empty(B.lazyllm_op_score_scratch_bytes(rows, H), dtype=torch.uint8, device=DEV)
        B.lazyllm_op_score(q_last, k, s_ref, scratch, rows, H, hd)
        s = torch.full((rows,), -2.0, dtype=torch.float32, device=DEV)
        # nothing allocated, neither through torch nor from the device behind its back (garbage of
        # earlier tests is collected first, so that nothing of theirs is freed in between)
        gc.collect()
        torch.cuda.synchronize()
        before, free_before = torch.cuda.memory_allocated(), torch.cuda.mem_get_info()[0]
        B.lazyllm_op_score_static(q_last, k, s, rows, H, hd)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        # (a scratch buffer would be megabytes.  Not on the first call of the process: the runtime
        # loads the code object that holds the static array then, and the array with it)
        assert call == 0 or free_before - torch.cuda.mem_get_info()[0] < (1 << 20)
        assert torch.equal(s, s_ref), rows           # same kernels, same order of operations
        want = O.last_row_scores(_f64(q_last).reshape(H, hd), _f64(k).reshape(rows, H, hd))
        got = s.cpu().numpy().astype(np.float64)
        assert np.allclose(got, want, rtol=2e-5, atol=1e-9), np.abs(got / want - 1).max()
        assert abs(got.sum() - 1.0) < 1e-5


def test_static_scratch_scoring_small_shapes_and_limits():
    rng = np.random.default_rng(78)
    for rows, H, hd in ((257, 4, 64), (1, 4, 64), (17, 32, 128)):
        k = _rand_bf16(rng, (rows, H * hd))
        q_last = _rand_bf16(rng, (H * hd,), 1.5)
        s = torch.full((rows,), -2.0, dtype=torch.float32, device=DEV)
        B.lazyllm_op_score_static(q_last, k, s, rows, H, hd)
        torch.cuda.synchronize()
        want = O.last_row_scores(_f64(q_last).reshape(H, hd), _f64(k).reshape(rows, H, hd))
        assert np.allclose(s.cpu().numpy().astype(np.float64), want, rtol=2e-5, atol=1e-9)
    # beyond the static array: refused before anything is launched
    H, hd = 64, 128
    rows = 40000
    assert B.lazyllm_op_score_scratch_bytes(rows, H) > 6 * 1024 * 1024
    k = torch.zeros(8, dtype=torch.bfloat16, device=DEV)      # never read
    s = torch.full((8,), -2.0, dtype=torch.float32, device=DEV)
    with pytest.raises(B.LazyLLMError) as e:
        B.lazyllm_op_score_static(k, k, s, rows, H, hd)
    assert e.value.status == B.LAZYLLM_ENOSPC
    torch.cuda.synchronize()
    assert float(s.min()) == -2.0
