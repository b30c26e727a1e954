"""ctypes binding of liblazyllm.so: same names as include/lazyllm.h, argument marshalling only.

Every step of the path runs inside the library's HIP kernels; torch is used for device
memory and for the stream handle.  There is no fallback: if the library is missing, the
first call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblazyllm.so")
MAX_LAYERS = 128

LAZYLLM_OK, LAZYLLM_EINVAL, LAZYLLM_ENOSPC, LAZYLLM_EHIP, LAZYLLM_ENOMEM, LAZYLLM_EFAILED = 0, -1, -2, -3, -4, -5
LAZYLLM_SCORE_ALL_LAYERS, LAZYLLM_SCORE_ONLY_USED, LAZYLLM_KEEP_HIDDEN, LAZYLLM_FUSE_COMPACTION = 0, 1, 2, 4
LAZYLLM_ST_BAD_TOKEN, LAZYLLM_ST_BAD_CU, LAZYLLM_ST_NO_STATE, LAZYLLM_ST_EXCHANGE = 1, 2, 4, 8
EPI_STORE, EPI_RESIDUAL, EPI_SWIGLU = 0, 1, 2


class lazyllm_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32),
                ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("n_kv_heads", C.c_int32),
                ("gemm_dtype", C.c_int32)]


class lazyllm_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p),
                ("attn_norm", C.POINTER(C.c_void_p)), ("wq", C.POINTER(C.c_void_p)),
                ("wk", C.POINTER(C.c_void_p)), ("wv", C.POINTER(C.c_void_p)),
                ("wo", C.POINTER(C.c_void_p)), ("ffn_norm", C.POINTER(C.c_void_p)),
                ("w_gate", C.POINTER(C.c_void_p)), ("w_up", C.POINTER(C.c_void_p)),
                ("w_down", C.POINTER(C.c_void_p)),
                ("final_norm", C.c_void_p), ("lm_head", C.c_void_p)]


class lazyllm_keep(C.Structure):
    _fields_ = [("layer", C.c_int32), ("keep_permille", C.c_int32)]


class lazyllm_result(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_layers", C.c_int32),
                ("n_tokens", C.c_int32 * MAX_LAYERS),
                ("logits", C.c_void_p),
                ("kept_pos", C.c_void_p * MAX_LAYERS), ("cu_kept", C.c_void_p * MAX_LAYERS),
                ("k", C.c_void_p * MAX_LAYERS), ("v", C.c_void_p * MAX_LAYERS),
                ("scores", C.c_void_p * MAX_LAYERS),
                ("n_aux", C.c_int32 * MAX_LAYERS),
                ("aux_h", C.c_void_p * MAX_LAYERS), ("aux_pos", C.c_void_p * MAX_LAYERS),
                ("cu_aux", C.c_void_p * MAX_LAYERS),
                ("status", C.c_void_p),
                ("hidden_in", C.c_void_p * MAX_LAYERS), ("hidden_out", C.c_void_p)]


class lazyllm_generation_view(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("capacity", C.c_int32), ("n_prompt", C.c_int32),
                ("n_tokens", C.c_int32), ("vt_ld", C.c_int32),
                ("k", C.c_void_p * MAX_LAYERS), ("vt", C.c_void_p * MAX_LAYERS),
                ("has_kv", C.c_void_p * MAX_LAYERS), ("aux_h", C.c_void_p * MAX_LAYERS),
                ("has_aux", C.c_void_p * MAX_LAYERS)]


class lazyllm_step_result(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_tokens", C.c_int32), ("position", C.c_int32),
                ("logits", C.c_void_p),
                ("n_selected", C.c_int32 * MAX_LAYERS), ("n_ran", C.c_int32 * MAX_LAYERS),
                ("selected", C.c_void_p * MAX_LAYERS), ("ran_pos", C.c_void_p * MAX_LAYERS),
                ("scores", C.c_void_p * MAX_LAYERS), ("status", C.c_void_p)]


class lazyllm_profile_record(C.Structure):
    _fields_ = [("step", C.c_int32), ("layer", C.c_int32), ("rows", C.c_int32), ("ms", C.c_float),
                ("work", C.c_double)]


STEP_NAMES = ("plan", "rope_table", "embed", "select", "gather", "rmsnorm", "gemm_qkv", "v_transpose",
              "score", "attention", "gemm_o", "gemm_gate_up", "gemm_down", "lm_head")

_lib_handle = None

_SIGNATURES = {
    "lazyllm_abi_version": (C.c_int, []),
    "lazyllm_strerror": (C.c_char_p, [C.c_int]),
    "lazyllm_last_hip_error": (C.c_int, []),
    "lazyllm_keep_counts": (C.c_int, [C.c_int32, C.c_int32, C.POINTER(lazyllm_keep), C.c_int32,
                                      C.POINTER(C.c_int32)]),
    "lazyllm_workspace_bytes": (C.c_size_t, [C.POINTER(lazyllm_config), C.c_int32, C.c_int32,
                                             C.c_int32]),
    "lazyllm_output_bytes": (C.c_size_t, [C.POINTER(lazyllm_config), C.POINTER(C.c_int32), C.c_int32,
                                          C.POINTER(lazyllm_keep), C.c_int32, C.c_uint32]),
    "lazyllm_model_create": (C.c_int, [C.POINTER(lazyllm_config), C.POINTER(lazyllm_weights),
                                       C.c_void_p, C.POINTER(C.c_void_p)]),
    "lazyllm_model_destroy": (None, [C.c_void_p]),
    "lazyllm_prefill": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                  C.POINTER(lazyllm_keep), C.c_int32, C.c_uint32, C.c_void_p,
                                  C.c_size_t, C.c_void_p, C.c_size_t, C.c_void_p,
                                  C.POINTER(lazyllm_result)]),
    "lazyllm_prefill_varlen": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_int32),
                                         C.c_void_p, C.c_int32, C.POINTER(lazyllm_keep), C.c_int32,
                                         C.c_uint32, C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t,
                                         C.c_void_p, C.POINTER(lazyllm_result)]),
    "lazyllm_generation_state_bytes": (C.c_size_t, [C.POINTER(lazyllm_config), C.POINTER(lazyllm_keep),
                                                    C.c_int32, C.c_int32]),
    "lazyllm_decode_workspace_bytes": (C.c_size_t, [C.POINTER(lazyllm_config), C.POINTER(lazyllm_keep),
                                                    C.c_int32, C.c_int32]),
    "lazyllm_generation_create": (C.c_int, [C.c_void_p, C.POINTER(lazyllm_keep), C.c_int32, C.c_int32,
                                            C.POINTER(lazyllm_result), C.c_void_p, C.c_size_t,
                                            C.c_void_p, C.POINTER(C.c_void_p)]),
    "lazyllm_generation_destroy": (None, [C.c_void_p]),
    "lazyllm_generation_get_view": (C.c_int, [C.c_void_p, C.POINTER(lazyllm_generation_view)]),
    "lazyllm_decode_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p,
                                      C.POINTER(lazyllm_step_result)]),
    "lazyllm_profile_begin": (C.c_int, []),
    "lazyllm_profile_end": (C.c_int, [C.POINTER(lazyllm_profile_record), C.c_int32,
                                      C.POINTER(C.c_int32)]),
    "lazyllm_op_gemm_workspace_bytes": (C.c_size_t, []),
    "lazyllm_op_gemm": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                  C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                  C.c_void_p, C.c_size_t, C.c_void_p]),
    "lazyllm_op_gemm_rmsnorm": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                          C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                          C.c_int32, C.c_void_p, C.c_float, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_size_t, C.c_void_p]),
    "lazyllm_op_pack_weight_stream": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                                C.c_void_p]),
    "lazyllm_op_pack_weight_ksteps": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                                C.c_void_p]),
    "lazyllm_op_quantize_fp8": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                          C.c_int32, C.c_void_p, C.c_void_p]),
    "lazyllm_op_gemm_fp8": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                      C.c_int32, C.c_int32, C.c_void_p]),
    "lazyllm_op_rmsnorm": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                     C.c_float, C.c_void_p]),
    "lazyllm_op_qkv_rope": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                      C.c_int32, C.c_float, C.c_void_p]),
    "lazyllm_op_v_transpose": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                         C.c_int32, C.c_void_p]),
    "lazyllm_op_attention": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                       C.c_int32, C.c_int32, C.c_int32, C.c_void_p]),
    "lazyllm_op_attention_score": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                             C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                             C.c_void_p]),
    "lazyllm_op_score_scratch_bytes": (C.c_size_t, [C.c_int32, C.c_int32]),
    "lazyllm_op_score": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                   C.c_int32, C.c_int32, C.c_void_p]),
    "lazyllm_op_score_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                          C.c_int32, C.c_void_p]),
    "lazyllm_op_select": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                    C.c_void_p]),
    "lazyllm_op_gather": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                    C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_int32, C.c_void_p]),
    "lazyllm_op_lm_head": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_int32, C.c_int32, C.c_float, C.c_void_p]),
}


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib_handle
    if _lib_handle is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "liblazyllm.so is not built (%s); run `python -m paper_2407_14057_amd.build`. "
                "There is no fallback path." % LIB_PATH)
        h = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(h, name)
            fn.restype = res
            fn.argtypes = args
        _lib_handle = h
    return _lib_handle


class LazyLLMError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        msg = lib().lazyllm_strerror(status).decode()
        if status == LAZYLLM_EHIP:
            msg += " (hipError_t %d)" % lib().lazyllm_last_hip_error()
        super().__init__("lazyllm: %s (%d)" % (msg, status))


def _check(status: int) -> None:
    if status != LAZYLLM_OK:
        raise LazyLLMError(status)


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, torch.Tensor):
        assert t.is_contiguous()
        return t.data_ptr()
    return int(t)


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream


def make_config(shape: Dict[str, float]) -> lazyllm_config:
    return lazyllm_config(int(shape["n_layers"]), int(shape["d_model"]), int(shape["n_heads"]),
                          int(shape["head_dim"]), int(shape["d_ffn"]), int(shape["vocab"]),
                          float(shape["rms_eps"]), float(shape["rope_theta"]),
                          int(shape.get("n_kv_heads", 0) or 0), int(shape.get("gemm_dtype", 0) or 0))


def _kv_heads(cfg: lazyllm_config) -> int:
    return cfg.n_kv_heads if cfg.n_kv_heads > 0 else cfg.n_heads


def make_schedule(schedule: Sequence[Tuple[int, int]]):
    arr = (lazyllm_keep * max(1, len(schedule)))()
    for i, (layer, permille) in enumerate(schedule):
        arr[i].layer = int(layer)
        arr[i].keep_permille = int(permille)
    return arr, len(schedule)


# ---------------------------------------------------------------------------- host-only helpers

def lazyllm_keep_counts(n: int, n_layers: int, schedule: Sequence[Tuple[int, int]]) -> List[int]:
    arr, ns = make_schedule(schedule)
    out = (C.c_int32 * max(1, n_layers))()
    _check(lib().lazyllm_keep_counts(n, n_layers, arr, ns, out))
    return [int(out[i]) for i in range(n_layers)]


def lazyllm_workspace_bytes(cfg: lazyllm_config, total_tokens: int, batch: int, max_seqlen: int) -> int:
    return int(lib().lazyllm_workspace_bytes(C.byref(cfg), total_tokens, batch, max_seqlen))


def lazyllm_output_bytes(cfg: lazyllm_config, seqlens: Sequence[int],
                         schedule: Sequence[Tuple[int, int]], flags: int = 0) -> int:
    arr, ns = make_schedule(schedule)
    sl = (C.c_int32 * len(seqlens))(*[int(x) for x in seqlens])
    return int(lib().lazyllm_output_bytes(C.byref(cfg), sl, len(seqlens), arr, ns, flags))


# ---------------------------------------------------------------------------- model + prefill

_PER_LAYER = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


def lazyllm_model_create(cfg: lazyllm_config, weights: Dict[str, object],
                         stream: Optional[torch.cuda.Stream] = None) -> int:
    """weights: {'embed','final_norm','lm_head': bf16 cuda tensors, per-layer names: lists}."""
    w = lazyllm_weights()
    keep = []
    for name in ("embed", "final_norm", "lm_head"):
        setattr(w, name, _ptr(weights[name]))
    for name in _PER_LAYER:
        arr = (C.c_void_p * cfg.n_layers)(*[_ptr(t) for t in weights[name]])
        keep.append(arr)
        setattr(w, name, C.cast(arr, C.POINTER(C.c_void_p)))
    out = C.c_void_p()
    _check(lib().lazyllm_model_create(C.byref(cfg), C.byref(w), _stream_ptr(stream), C.byref(out)))
    return out.value


def lazyllm_model_destroy(model: int) -> None:
    lib().lazyllm_model_destroy(model)


def lazyllm_prefill(model: int, token_ids, embed_scale, n: int, schedule, flags: int, workspace,
                    out_buf, stream: Optional[torch.cuda.Stream] = None) -> lazyllm_result:
    arr, ns = make_schedule(schedule)
    res = lazyllm_result()
    _check(lib().lazyllm_prefill(model, _ptr(token_ids), _ptr(embed_scale), n, arr, ns, flags,
                                 _ptr(workspace), workspace.numel() * workspace.element_size(),
                                 _ptr(out_buf), out_buf.numel() * out_buf.element_size(),
                                 _stream_ptr(stream), C.byref(res)))
    return res


def lazyllm_prefill_varlen(model: int, token_ids, embed_scale, cu_seqlens_host: Sequence[int],
                           cu_seqlens_dev, schedule, flags: int, workspace, out_buf,
                           stream: Optional[torch.cuda.Stream] = None) -> lazyllm_result:
    arr, ns = make_schedule(schedule)
    res = lazyllm_result()
    batch = len(cu_seqlens_host) - 1
    cu = (C.c_int32 * (batch + 1))(*[int(x) for x in cu_seqlens_host])
    _check(lib().lazyllm_prefill_varlen(model, _ptr(token_ids), _ptr(embed_scale), cu,
                                        _ptr(cu_seqlens_dev), batch, arr, ns, flags,
                                        _ptr(workspace), workspace.numel() * workspace.element_size(),
                                        _ptr(out_buf), out_buf.numel() * out_buf.element_size(),
                                        _stream_ptr(stream), C.byref(res)))
    return res


def lazyllm_profile_begin() -> None:
    _check(lib().lazyllm_profile_begin())


def lazyllm_profile_end(capacity: int = 65536) -> List[Dict[str, float]]:
    buf = (lazyllm_profile_record * capacity)()
    n = C.c_int32(0)
    _check(lib().lazyllm_profile_end(buf, capacity, C.byref(n)))
    return [dict(step=STEP_NAMES[buf[i].step], layer=int(buf[i].layer), rows=int(buf[i].rows),
                 ms=float(buf[i].ms), work=float(buf[i].work)) for i in range(min(n.value, capacity))]


# ---------------------------------------------------------------------------- single steps

def lazyllm_op_gemm_workspace_bytes() -> int:
    return int(lib().lazyllm_op_gemm_workspace_bytes())


def lazyllm_op_gemm(A, W, Cout, R, M, N, K, lda, ldw, ldc, epilogue, stream=None, workspace=None) -> None:
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lazyllm_op_gemm(_ptr(A), _ptr(W), _ptr(Cout), _ptr(R), M, N, K, lda, ldw, ldc,
                                 epilogue, _ptr(workspace), wsb, _stream_ptr(stream)))


def lazyllm_op_gemm_rmsnorm(A, W, Cout, R, M, N, K, lda, ldw, ldc, epilogue, ssq_in=None, eps=1e-5,
                            ssq_out=None, ssq_clear=None, stream=None, workspace=None) -> None:
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lazyllm_op_gemm_rmsnorm(_ptr(A), _ptr(W), _ptr(Cout), _ptr(R), M, N, K, lda, ldw, ldc,
                                         epilogue, _ptr(ssq_in), eps, _ptr(ssq_out), _ptr(ssq_clear),
                                         _ptr(workspace), wsb, _stream_ptr(stream)))


def lazyllm_op_pack_weight_stream(W, N, K, ldw, packed, stream=None) -> None:
    _check(lib().lazyllm_op_pack_weight_stream(_ptr(W), N, K, ldw, _ptr(packed), _stream_ptr(stream)))


def lazyllm_op_pack_weight_ksteps(W, N, K, ldw, packed, stream=None) -> None:
    _check(lib().lazyllm_op_pack_weight_ksteps(_ptr(W), N, K, ldw, _ptr(packed), _stream_ptr(stream)))


def lazyllm_op_quantize_fp8(x, rows, K, ldx, codes, ldq, scale, stream=None) -> None:
    _check(lib().lazyllm_op_quantize_fp8(_ptr(x), rows, K, ldx, _ptr(codes), ldq, _ptr(scale),
                                         _stream_ptr(stream)))


def lazyllm_op_gemm_fp8(a_codes, a_scale, w_codes, w_scale, Cout, R, M, N, K, lda, ldw, ldc, epilogue,
                        stream=None) -> None:
    _check(lib().lazyllm_op_gemm_fp8(_ptr(a_codes), _ptr(a_scale), _ptr(w_codes), _ptr(w_scale),
                                     _ptr(Cout), _ptr(R), M, N, K, lda, ldw, ldc, epilogue,
                                     _stream_ptr(stream)))


def lazyllm_op_rmsnorm(h, gain, x, rows, d, eps, stream=None) -> None:
    _check(lib().lazyllm_op_rmsnorm(_ptr(h), _ptr(gain), _ptr(x), rows, d, eps, _stream_ptr(stream)))


def lazyllm_op_qkv_rope(x, wqkv, pos, max_pos, rope_table, q, k, v, rows, n_heads, head_dim, theta,
                        stream=None) -> None:
    _check(lib().lazyllm_op_qkv_rope(_ptr(x), _ptr(wqkv), _ptr(pos), max_pos, _ptr(rope_table),
                                     _ptr(q), _ptr(k), _ptr(v), rows, n_heads, head_dim, theta,
                                     _stream_ptr(stream)))


def lazyllm_op_v_transpose(v, vt, vt_ld, rows, n_heads, head_dim, stream=None) -> None:
    _check(lib().lazyllm_op_v_transpose(_ptr(v), _ptr(vt), vt_ld, rows, n_heads, head_dim,
                                        _stream_ptr(stream)))


def lazyllm_op_attention(q, k, vt, vt_ld, o, rows, n_heads, head_dim, stream=None) -> None:
    _check(lib().lazyllm_op_attention(_ptr(q), _ptr(k), _ptr(vt), vt_ld, _ptr(o), rows, n_heads,
                                      head_dim, _stream_ptr(stream)))


def lazyllm_op_attention_score(q, k, vt, vt_ld, o, s, scratch, rows, n_heads, head_dim,
                               stream=None) -> None:
    _check(lib().lazyllm_op_attention_score(_ptr(q), _ptr(k), _ptr(vt), vt_ld, _ptr(o), _ptr(s),
                                            _ptr(scratch), rows, n_heads, head_dim,
                                            _stream_ptr(stream)))


def lazyllm_op_score_scratch_bytes(rows: int, n_heads: int) -> int:
    return int(lib().lazyllm_op_score_scratch_bytes(rows, n_heads))


def lazyllm_op_score(q_last, k, s, scratch, rows, n_heads, head_dim, stream=None) -> None:
    _check(lib().lazyllm_op_score(_ptr(q_last), _ptr(k), _ptr(s), _ptr(scratch), rows, n_heads,
                                  head_dim, _stream_ptr(stream)))


def lazyllm_op_score_static(q_last, k, s, rows, n_heads, head_dim, stream=None) -> None:
    _check(lib().lazyllm_op_score_static(_ptr(q_last), _ptr(k), _ptr(s), rows, n_heads, head_dim,
                                         _stream_ptr(stream)))


def lazyllm_op_select(s, m, k, keep_idx, prune_idx, stream=None) -> None:
    _check(lib().lazyllm_op_select(_ptr(s), m, k, _ptr(keep_idx), _ptr(prune_idx),
                                   _stream_ptr(stream)))


def lazyllm_op_gather(h, pos, keep_idx, n_keep, prune_idx, n_prune, h_out, pos_out, aux_h, aux_pos,
                      d, stream=None) -> None:
    _check(lib().lazyllm_op_gather(_ptr(h), _ptr(pos), _ptr(keep_idx), n_keep, _ptr(prune_idx),
                                   n_prune, _ptr(h_out), _ptr(pos_out), _ptr(aux_h), _ptr(aux_pos),
                                   d, _stream_ptr(stream)))


def lazyllm_op_lm_head(h_last, gain, w_lm, xf, logits, d, vocab, eps, stream=None) -> None:
    _check(lib().lazyllm_op_lm_head(_ptr(h_last), _ptr(gain), _ptr(w_lm), _ptr(xf), _ptr(logits), d,
                                    vocab, eps, _stream_ptr(stream)))


# ---------------------------------------------------------------------------- decoding steps

def lazyllm_generation_state_bytes(cfg: lazyllm_config, schedule, capacity: int) -> int:
    arr, ns = make_schedule(schedule)
    return int(lib().lazyllm_generation_state_bytes(C.byref(cfg), arr, ns, capacity))


def lazyllm_decode_workspace_bytes(cfg: lazyllm_config, schedule, capacity: int) -> int:
    arr, ns = make_schedule(schedule)
    return int(lib().lazyllm_decode_workspace_bytes(C.byref(cfg), arr, ns, capacity))


def lazyllm_generation_create(model: int, schedule, capacity: int, prefill: lazyllm_result, state,
                              stream=None) -> int:
    arr, ns = make_schedule(schedule)
    handle = C.c_void_p()
    _check(lib().lazyllm_generation_create(model, arr, ns, capacity, C.byref(prefill), _ptr(state),
                                           state.numel() if state is not None else 0,
                                           _stream_ptr(stream), C.byref(handle)))
    return handle.value


def lazyllm_generation_destroy(handle: int) -> None:
    lib().lazyllm_generation_destroy(handle)


def lazyllm_generation_get_view(handle: int) -> lazyllm_generation_view:
    v = lazyllm_generation_view()
    _check(lib().lazyllm_generation_get_view(handle, C.byref(v)))
    return v


def lazyllm_decode_step(handle: int, token_id, workspace, stream=None) -> lazyllm_step_result:
    res = lazyllm_step_result()
    _check(lib().lazyllm_decode_step(handle, _ptr(token_id), _ptr(workspace),
                                     workspace.numel() if workspace is not None else 0,
                                     _stream_ptr(stream), C.byref(res)))
    return res


# ---------------------------------------------------------------------------- result views

class PrefillOutput:
    """Zero-copy torch views of a lazyllm_result (all data stays in `out_buf`)."""

    def __init__(self, res: lazyllm_result, out_buf: torch.Tensor, cfg: lazyllm_config):
        self.res, self.out_buf, self.cfg = res, out_buf, cfg
        self.batch, self.n_layers = res.batch, res.n_layers
        self.n_tokens = [int(res.n_tokens[l]) for l in range(res.n_layers)]
        self.n_aux = [int(res.n_aux[l]) for l in range(res.n_layers)]

    def _view(self, ptr: Optional[int], count: int, dtype: torch.dtype) -> Optional[torch.Tensor]:
        if not ptr:
            return None
        off = ptr - self.out_buf.data_ptr()
        nbytes = count * torch.empty((), dtype=dtype).element_size()
        return self.out_buf[off: off + nbytes].view(dtype)

    @property
    def logits(self):
        return self._view(self.res.logits, self.batch * self.cfg.vocab, torch.float32).view(
            self.batch, self.cfg.vocab)

    @property
    def status(self) -> int:
        return int(self._view(self.res.status, 1, torch.int32).item())

    def kept_pos(self, l):
        return self._view(self.res.kept_pos[l], self.n_tokens[l], torch.int32)

    def cu_kept(self, l):
        return self._view(self.res.cu_kept[l], self.batch + 1, torch.int32)

    def k(self, l):
        hkv, hd = _kv_heads(self.cfg), self.cfg.head_dim
        return self._view(self.res.k[l], self.n_tokens[l] * hkv * hd, torch.bfloat16).view(
            self.n_tokens[l], hkv, hd)

    def v(self, l):
        hkv, hd = _kv_heads(self.cfg), self.cfg.head_dim
        return self._view(self.res.v[l], self.n_tokens[l] * hkv * hd, torch.bfloat16).view(
            self.n_tokens[l], hkv, hd)

    def scores(self, l):
        return self._view(self.res.scores[l], self.n_tokens[l], torch.float32)

    def aux_h(self, l):
        if not self.res.aux_h[l]:
            return None
        return self._view(self.res.aux_h[l], self.n_aux[l] * self.cfg.d_model, torch.bfloat16).view(
            self.n_aux[l], self.cfg.d_model)

    def aux_pos(self, l):
        if not self.res.aux_pos[l]:
            return None
        return self._view(self.res.aux_pos[l], self.n_aux[l], torch.int32)

    def cu_aux(self, l):
        return self._view(self.res.cu_aux[l], self.batch + 1, torch.int32)

    def hidden_in(self, l):
        if not self.res.hidden_in[l]:
            return None
        return self._view(self.res.hidden_in[l], self.n_tokens[l] * self.cfg.d_model,
                          torch.bfloat16).view(self.n_tokens[l], self.cfg.d_model)

    @property
    def hidden_out(self):
        if not self.res.hidden_out:
            return None
        n = self.n_tokens[self.n_layers - 1]
        return self._view(self.res.hidden_out, n * self.cfg.d_model, torch.bfloat16).view(n, self.cfg.d_model)


class Model:
    """Owns a lazyllm_model handle and reusable workspace / output buffers."""

    def __init__(self, shape: Dict[str, float], weights: Dict[str, object], device: str = "cuda:0"):
        self.cfg = make_config(shape)
        self.device = torch.device(device)
        with torch.cuda.device(self.device):
            self.handle = lazyllm_model_create(self.cfg, weights)
        self._ws = None
        self._out = None

    def close(self) -> None:
        if self.handle:
            lazyllm_model_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def buffers(self, seqlens: Sequence[int], schedule, flags: int = 0) -> Tuple[torch.Tensor, torch.Tensor]:
        total, batch, mx = int(sum(seqlens)), len(seqlens), int(max(seqlens))
        wsb = lazyllm_workspace_bytes(self.cfg, total, batch, mx)
        outb = lazyllm_output_bytes(self.cfg, seqlens, schedule, flags)
        if wsb == 0 or outb == 0:
            raise LazyLLMError(LAZYLLM_EINVAL)
        if self._ws is None or self._ws.numel() < wsb:
            self._ws = torch.empty(wsb, dtype=torch.uint8, device=self.device)
        if self._out is None or self._out.numel() < outb:
            self._out = torch.empty(outb, dtype=torch.uint8, device=self.device)
        return self._ws, self._out

    def prefill(self, token_ids: torch.Tensor, schedule, *, cu_seqlens: Optional[Sequence[int]] = None,
                embed_scale: Optional[torch.Tensor] = None, flags: int = 0,
                stream: Optional[torch.cuda.Stream] = None) -> PrefillOutput:
        """token_ids: int32 cuda tensor (all prompts packed).  Asynchronous on the stream."""
        if cu_seqlens is None:
            cu_seqlens = [0, int(token_ids.numel())]
        seqlens = [int(cu_seqlens[i + 1] - cu_seqlens[i]) for i in range(len(cu_seqlens) - 1)]
        ws, out = self.buffers(seqlens, schedule, flags)
        if len(seqlens) == 1:
            res = lazyllm_prefill(self.handle, token_ids, embed_scale, seqlens[0], schedule, flags,
                                  ws, out, stream)
        else:
            cu_dev = torch.tensor([int(x) for x in cu_seqlens], dtype=torch.int32, device=self.device)
            self._cu_dev = cu_dev
            res = lazyllm_prefill_varlen(self.handle, token_ids, embed_scale, cu_seqlens, cu_dev,
                                         schedule, flags, ws, out, stream)
        return PrefillOutput(res, out, self.cfg)


def _buf_view(buf: torch.Tensor, ptr: Optional[int], count: int, dtype: torch.dtype):
    if not ptr:
        return None
    off = ptr - buf.data_ptr()
    nbytes = count * torch.empty((), dtype=dtype).element_size()
    return buf[off: off + nbytes].view(dtype)


class StepOutput:
    """Zero-copy torch views of a lazyllm_step_result."""

    def __init__(self, res: lazyllm_step_result, state: torch.Tensor, ws: torch.Tensor, cfg: lazyllm_config):
        self.res, self.state, self.ws, self.cfg = res, state, ws, cfg
        self.n_layers, self.n_tokens, self.position = res.n_layers, res.n_tokens, res.position
        self.n_selected = [int(res.n_selected[l]) for l in range(res.n_layers)]
        self.n_ran = [int(res.n_ran[l]) for l in range(res.n_layers)]

    @property
    def logits(self):
        return _buf_view(self.state, self.res.logits, self.cfg.vocab, torch.float32)

    @property
    def status(self) -> int:
        return int(_buf_view(self.state, self.res.status, 1, torch.int32).item())

    def selected(self, l):
        """uint8 [n_tokens] membership by position, or None when every token is selected."""
        return _buf_view(self.ws, self.res.selected[l], self.n_tokens, torch.uint8)

    def ran_pos(self, l):
        return _buf_view(self.ws, self.res.ran_pos[l], self.n_ran[l], torch.int32)

    def scores(self, l):
        return _buf_view(self.ws, self.res.scores[l], self.n_tokens, torch.float32)


class Generation:
    """Owns the state buffer, the step workspace and the handle of one sequence's decoding."""

    def __init__(self, model: Model, schedule, prefill: PrefillOutput, capacity: int,
                 stream: Optional[torch.cuda.Stream] = None):
        self.model, self.cfg, self.schedule = model, model.cfg, list(schedule)
        sb = lazyllm_generation_state_bytes(self.cfg, schedule, capacity)
        wb = lazyllm_decode_workspace_bytes(self.cfg, schedule, capacity)
        if sb == 0 or wb == 0:
            raise LazyLLMError(LAZYLLM_EINVAL)
        self.state = torch.empty(sb, dtype=torch.uint8, device=model.device)
        self.ws = torch.empty(wb, dtype=torch.uint8, device=model.device)
        self.handle = lazyllm_generation_create(model.handle, schedule, capacity, prefill.res, self.state,
                                                stream)

    def close(self) -> None:
        if self.handle:
            lazyllm_generation_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def step(self, token_id: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> StepOutput:
        """token_id: int32 cuda tensor with one element."""
        res = lazyllm_decode_step(self.handle, token_id, self.ws, stream)
        return StepOutput(res, self.state, self.ws, self.cfg)

    def view(self):
        """{'k': [..], 'vt': [..], 'has_kv': [..], 'aux_h': [..], 'has_aux': [..]} torch views by layer."""
        v = lazyllm_generation_get_view(self.handle)
        cap, d, ld = v.capacity, self.cfg.d_model, v.vt_ld
        kvd = _kv_heads(self.cfg) * self.cfg.head_dim
        out = {"n_tokens": v.n_tokens, "capacity": cap, "vt_ld": ld, "k": [], "vt": [], "has_kv": [],
               "aux_h": [], "has_aux": []}
        for l in range(v.n_layers):
            out["k"].append(_buf_view(self.state, v.k[l], cap * kvd, torch.bfloat16).view(cap, kvd))
            out["vt"].append(_buf_view(self.state, v.vt[l], kvd * ld, torch.bfloat16).view(kvd, ld))
            out["has_kv"].append(_buf_view(self.state, v.has_kv[l], cap, torch.uint8))
            a = _buf_view(self.state, v.aux_h[l], cap * d, torch.bfloat16)
            out["aux_h"].append(None if a is None else a.view(cap, d))
            out["has_aux"].append(_buf_view(self.state, v.has_aux[l], cap, torch.uint8))
        return out
