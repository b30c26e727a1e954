"""Host-side checks that need no GPU: the library loads, exports what the header declares,
and rejects bad arguments before any HIP call."""
import os
import re

import numpy as np
import pytest

from oracle import lazyllm_oracle as O
from paper_2407_14057_amd import binding as B
from paper_2407_14057_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "lazyllm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lazyllm_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    names = _declared_symbols()
    assert len(names) >= 22
    assert lib.lazyllm_op_gemm_workspace_bytes() > 0
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(B._SIGNATURES), "binding and header disagree"
    assert lib.lazyllm_abi_version() == 3
    assert lib.lazyllm_strerror(-1) == b"invalid argument"
    assert lib.lazyllm_strerror(-2) == b"workspace or output buffer too small"
    assert lib.lazyllm_strerror(-5).startswith(b"generation handle unusable")


def test_binding_constants_are_the_headers():
    """Every status code, flag and status bit the header defines has the same value in the binding."""
    text = open(os.path.join(ROOT, "include", "lazyllm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    found = {n: int(v.rstrip("u")) for n, v in re.findall(r"#define\s+(LAZYLLM_\w+)\s+(-?\d+u?)\b", text)}
    found.update({n: int(v) for n, v in re.findall(r"\b(LAZYLLM_E?\w+)\s*=\s*(-?\d+)", text)})
    for name in ("LAZYLLM_OK", "LAZYLLM_EINVAL", "LAZYLLM_ENOSPC", "LAZYLLM_EHIP", "LAZYLLM_ENOMEM", "LAZYLLM_EFAILED",
                 "LAZYLLM_SCORE_ONLY_USED", "LAZYLLM_KEEP_HIDDEN", "LAZYLLM_FUSE_COMPACTION", "LAZYLLM_ST_BAD_TOKEN", "LAZYLLM_ST_BAD_CU",
                 "LAZYLLM_ST_NO_STATE", "LAZYLLM_ST_EXCHANGE"):
        assert name in found, name
        assert getattr(B, name) == found[name], name
    assert found["LAZYLLM_MAX_LAYERS"] == B.MAX_LAYERS
    # the status bits are distinct single bits
    bits = [found[n] for n in found if n.startswith("LAZYLLM_ST_")]
    assert len(bits) == 4 and all(b & (b - 1) == 0 for b in bits) and len(set(bits)) == 4


def test_keep_counts_match_checker():
    cases = [(512, 4, [(2, 700), (3, 500)]), (3376, 32, [(8, 700), (16, 500), (24, 300)]),
             (8192, 32, [(8, 600), (16, 400), (24, 200)]), (3376, 32, [(4, 500), (12, 500), (20, 500)]),
             (10, 3, [(1, 600)]), (1, 5, [(1, 1), (4, 1)]), (7, 4, [(1, 1000), (2, 1)])]
    rng = np.random.default_rng(0)
    for _ in range(50):
        L = int(rng.integers(2, 40))
        layers = sorted(rng.choice(np.arange(1, L), size=min(L - 1, int(rng.integers(1, 5))), replace=False))
        cases.append((int(rng.integers(1, 100000)), L, [(int(l), int(rng.integers(1, 1001))) for l in layers]))
    for n, L, sched in cases:
        assert B.lazyllm_keep_counts(n, L, sched) == O.keep_counts(n, L, sched)


def test_bad_schedules_are_rejected():
    bad = [[(0, 500)],            # layer 0 has no prior scores
           [(4, 500)],            # layer out of range for L = 4
           [(2, 500), (1, 500)],  # unsorted
           [(2, 500), (2, 400)],  # duplicate
           [(1, 0)], [(1, 1001)], [(1, -5)]]
    for sched in bad:
        with pytest.raises(B.LazyLLMError) as e:
            B.lazyllm_keep_counts(100, 4, sched)
        assert e.value.status == B.LAZYLLM_EINVAL
        assert B.lazyllm_output_bytes(B.make_config(synth.TINY.as_dict()), [100], sched) == 0
    with pytest.raises(B.LazyLLMError):
        B.lazyllm_keep_counts(0, 4, [])


def test_sizes_are_positive_and_monotone():
    cfg = B.make_config(synth.TINY.as_dict())
    w1 = B.lazyllm_workspace_bytes(cfg, 512, 1, 512)
    w2 = B.lazyllm_workspace_bytes(cfg, 1024, 2, 512)
    assert 0 < w1 < w2
    o_dense = B.lazyllm_output_bytes(cfg, [512], [])
    o_pruned = B.lazyllm_output_bytes(cfg, [512], [(2, 700), (3, 500)])
    assert o_dense > 0 and o_pruned > 0
    # K/V of layer l hold exactly the tokens that ran it
    kv = lambda counts: sum(2 * n * cfg.d_model * 2 for n in counts)
    assert o_dense >= kv([512] * 4) and o_pruned >= kv([512, 512, 359, 180])
    assert o_pruned < o_dense + 512 * cfg.d_model * 2 + 65536
    # unsupported shapes
    bad = dict(synth.TINY.as_dict())
    bad["head_dim"] = 96
    assert B.lazyllm_workspace_bytes(B.make_config(bad), 512, 1, 512) == 0
    bad = dict(synth.TINY.as_dict())
    bad["n_heads"] = 3
    assert B.lazyllm_workspace_bytes(B.make_config(bad), 512, 1, 512) == 0
    assert B.lazyllm_workspace_bytes(cfg, 0, 1, 1) == 0
    assert B.lazyllm_workspace_bytes(cfg, 10, 1, 11) == 0
    assert B.lazyllm_output_bytes(cfg, [0], []) == 0
    # shared K,V heads: the count must divide the heads and keep the K,V width a multiple of 128
    gqa = dict(synth.TINY.as_dict())
    gqa["n_kv_heads"] = 2
    cfg2 = B.make_config(gqa)
    assert B.lazyllm_workspace_bytes(cfg2, 512, 1, 512) > 0
    assert 0 < B.lazyllm_output_bytes(cfg2, [512], []) < o_dense          # K,V are half as wide
    for bad_kv in (3, 1, 5, -1):                   # 3 does not divide 4; 1 x 64 is not a multiple of 128
        gqa["n_kv_heads"] = bad_kv
        assert B.lazyllm_workspace_bytes(B.make_config(gqa), 512, 1, 512) == 0, bad_kv
    # 8-bit projections: a larger workspace (codes and scales of the activations); shapes whose
    # widths are not multiples of 256 and unknown arithmetic codes are refused
    f8 = dict(synth.TINY.as_dict())
    f8["gemm_dtype"] = 1
    assert B.lazyllm_workspace_bytes(B.make_config(f8), 512, 1, 512) > w1
    assert B.lazyllm_workspace_bytes(B.make_config(synth.TINY_FP8.as_dict()), 512, 1, 512) > w1
    f8["d_model"], f8["n_heads"] = 384, 6
    assert B.lazyllm_workspace_bytes(B.make_config(f8), 512, 1, 512) == 0
    f8 = dict(synth.TINY.as_dict())
    f8["gemm_dtype"] = 2
    assert B.lazyllm_workspace_bytes(B.make_config(f8), 512, 1, 512) == 0


def test_null_arguments_return_einval_without_touching_the_gpu():
    lib = B.lib()
    res = B.lazyllm_result()
    import ctypes as C
    arr, ns = B.make_schedule([(1, 500)])
    assert lib.lazyllm_prefill(None, None, None, 16, arr, ns, 0, None, 0, None, 0, None, C.byref(res)) == B.LAZYLLM_EINVAL
    assert lib.lazyllm_op_gemm(None, None, None, None, 1, 128, 64, 64, 64, 128, 0, None, 0, None) == B.LAZYLLM_EINVAL
    assert lib.lazyllm_op_gemm(1, 1, 1, None, 4, 100, 64, 64, 64, 100, 0, None, 0, None) == B.LAZYLLM_EINVAL   # N % 128
    assert lib.lazyllm_op_gemm(1, 1, 1, None, 4, 128, 60, 64, 64, 128, 0, None, 0, None) == B.LAZYLLM_EINVAL   # K % 64
    assert lib.lazyllm_op_gemm(1, 1, 1, None, 4, 128, 64, 64, 64, 128, 1, None, 0, None) == B.LAZYLLM_EINVAL   # residual w/o R
    assert lib.lazyllm_op_select(1, 10, 0, 1, 1, None) == B.LAZYLLM_EINVAL
    assert lib.lazyllm_op_select(1, 10, 11, 1, 1, None) == B.LAZYLLM_EINVAL
    assert lib.lazyllm_op_attention(1, 1, 1, 100, 1, 10, 4, 64, None) == B.LAZYLLM_EINVAL             # vt_ld % 64
    assert lib.lazyllm_op_attention(1, 1, 1, 128, 1, 10, 4, 96, None) == B.LAZYLLM_EINVAL             # head_dim
    assert lib.lazyllm_op_score(1, 1, 1, 1, 0, 4, 64, None) == B.LAZYLLM_EINVAL
    assert lib.lazyllm_op_score_scratch_bytes(0, 4) == 0
    assert lib.lazyllm_model_create(None, None, None, None) == B.LAZYLLM_EINVAL
    # the 8-bit variant's steps and the weight re-ordering steps
    assert lib.lazyllm_op_quantize_fp8(None, 4, 64, 64, None, 64, None, None) == B.LAZYLLM_EINVAL
    assert lib.lazyllm_op_quantize_fp8(16, 4, 60, 64, 16, 64, 16, None) == B.LAZYLLM_EINVAL            # K % 8
    assert lib.lazyllm_op_quantize_fp8(16, 4, 16392, 16392, 16, 16392, 16, None) == B.LAZYLLM_EINVAL   # K > 16384
    assert lib.lazyllm_op_gemm_fp8(None, None, None, None, None, None, 4, 256, 128, 128, 128, 256, 0, None) == B.LAZYLLM_EINVAL
    assert lib.lazyllm_op_gemm_fp8(16, 16, 16, 16, 16, None, 4, 128, 128, 128, 128, 128, 0, None) == B.LAZYLLM_EINVAL   # N % 256
    assert lib.lazyllm_op_gemm_fp8(16, 16, 16, 16, 16, None, 4, 256, 64, 64, 64, 256, 0, None) == B.LAZYLLM_EINVAL      # K % 128
    assert lib.lazyllm_op_gemm_fp8(16, 16, 16, 16, 16, None, 4, 256, 128, 128, 128, 256, 1, None) == B.LAZYLLM_EINVAL   # residual w/o R
    assert lib.lazyllm_op_gemm_fp8(24, 16, 16, 16, 16, None, 4, 256, 128, 128, 128, 256, 0, None) == B.LAZYLLM_EINVAL   # alignment
    assert lib.lazyllm_op_pack_weight_ksteps(None, 128, 64, 64, None, None) == B.LAZYLLM_EINVAL
    assert lib.lazyllm_op_pack_weight_ksteps(16, 128, 100, 104, 16, None) == B.LAZYLLM_EINVAL         # K % 64
    assert lib.lazyllm_op_pack_weight_stream(16, 100, 64, 64, 16, None) == B.LAZYLLM_EINVAL           # N % 128
    assert lib.lazyllm_op_pack_weight_stream(16, 128, 64, 32, 16, None) == B.LAZYLLM_EINVAL           # stride below K


def test_static_scratch_scoring_validates_before_any_hip_call():
    """The allocation-free Eq. 1 entry point rejects bad arguments and sizes beyond its static
    scratch on the host (no GPU here: reaching a HIP call would fail differently)."""
    lib = B.lib()
    one = 4096
    assert lib.lazyllm_op_score_static(None, one, one, 10, 4, 64, None) == B.LAZYLLM_EINVAL
    assert lib.lazyllm_op_score_static(one, one, one, 0, 4, 64, None) == B.LAZYLLM_EINVAL
    assert lib.lazyllm_op_score_static(one, one, one, 10, 4, 96, None) == B.LAZYLLM_EINVAL
    assert lib.lazyllm_op_score_static(one, one, one, 40000, 64, 128, None) == B.LAZYLLM_ENOSPC
    # the limit is the scratch size the buffer form would ask for
    assert B.lazyllm_op_score_scratch_bytes(39000, 32) <= 6 * 1024 * 1024 < B.lazyllm_op_score_scratch_bytes(40000, 32)
    assert lib.lazyllm_op_score_static(one, one, one, 40000, 32, 128, None) == B.LAZYLLM_ENOSPC


def test_bench_refuses_more_than_one_gpu():
    """One GPU is the whole target: `bench.py --gpus N` with N above 1 says so and exits non-zero,
    before anything touches a device."""
    import subprocess, sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
