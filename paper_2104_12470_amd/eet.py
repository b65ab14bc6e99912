"""Thin ctypes binding over libeet.so (the C ABI declared in include/eet.h).

Argument marshalling only: every computation runs in the HIP kernels of the library.  torch is
used for device memory and streams.  There is no fallback: if the library has not been built
(`python -m paper_2104_12470_amd.build`), loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libeet.so")

EET_OK = 0
EET_ERR_INVALID_ARG = -1
EET_ERR_UNSUPPORTED_SHAPE = -2
EET_ERR_CAPACITY = -3
EET_ERR_STATE = -4
EET_ERR_HIP = -5
EET_MAX_BATCH = 128

WEIGHT_FIELDS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                 "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


class LayerConfig(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("heads", C.c_int32), ("ffn", C.c_int32),
                ("max_batch", C.c_int32), ("max_prompt", C.c_int32), ("max_seq", C.c_int32),
                ("ln_eps", C.c_float)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_FIELDS]


class BufMgrStats(C.Structure):
    _fields_ = [("arena_bytes", C.c_uint64), ("footprint_bytes", C.c_uint64), ("buffers", C.c_int64), ("idle", C.c_int64),
                ("requests", C.c_int64), ("reused_same_size", C.c_int64), ("reused_larger", C.c_int64),
                ("created", C.c_int64)]


class ModelConfig(C.Structure):
    _fields_ = [("vocab", C.c_int32), ("vocab_padded", C.c_int32), ("max_pos", C.c_int32)]


MODEL_WEIGHT_FIELDS = ("wte", "wpe", "lnf_g", "lnf_b")


class ModelWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in MODEL_WEIGHT_FIELDS]


class EETError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"eet error {code}: {message}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2104_12470_amd.build` "
                               "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_size_t
        cfgp, i32p = C.POINTER(LayerConfig), C.POINTER(C.c_int32)
        sig = {
            "eet_kv_cache_bytes": (sz, [cfgp]),
            "eet_workspace_bytes": (sz, [cfgp]),
            "eet_layer_create": (i32, [cfgp, C.POINTER(LayerWeights), vp, C.POINTER(vp)]),
            "eet_prefill": (i32, [vp, i32p, i32, i32, vp, vp, vp, vp]),
            "eet_prefill_left_padded": (i32, [vp, i32p, i32, i32, vp, vp, vp, vp]),
            "eet_layer_encode": (i32, [vp, i32p, i32, i32, vp, vp, vp, vp]),
            "eet_decode_step": (i32, [vp, vp, vp, vp, vp]),
            "eet_cache_lens": (i32, [vp, i32p, vp]),
            "eet_restore": (i32, [vp, i32p, i32, vp]),
            "eet_stack_restore": (i32, [vp, i32p, i32, vp]),
            "eet_layer_destroy": (i32, [vp]),
            "eet_last_error": (C.c_char_p, []),
            "eet_stack_kv_cache_bytes": (sz, [cfgp, i32]),
            "eet_stack_workspace_bytes": (sz, [cfgp, i32]),
            "eet_stack_create": (i32, [cfgp, i32, C.POINTER(LayerWeights), vp, i32, C.POINTER(vp)]),
            "eet_stack_prefill": (i32, [vp, i32p, i32, i32, vp, vp, vp, vp]),
            "eet_stack_prefill_left_padded": (i32, [vp, i32p, i32, i32, vp, vp, vp, vp]),
            "eet_stack_encode": (i32, [vp, i32p, i32, i32, vp, vp, vp, vp]),
            "eet_stack_decode_step": (i32, [vp, vp, vp, vp, vp]),
            "eet_stack_cache_lens": (i32, [vp, i32p, vp]),
            "eet_stack_destroy": (i32, [vp]),
            "eet_op_layernorm": (i32, [vp, vp, vp, vp, i64, i32, f32, vp]),
            "eet_op_softmax_maskfree": (i32, [vp, i32p, i32, i32, i32, f32, vp]),
            "eet_op_softmax_maskfree_left_padded": (i32, [vp, i32p, i32, i32, i32, f32, vp]),
            "eet_op_bias_gelu": (i32, [vp, vp, vp, i64, i32, vp]),
            "eet_op_bias_residual": (i32, [vp, vp, vp, vp, i64, i32, vp]),
            "eet_op_linear": (i32, [vp, vp, vp, vp, vp, i64, i32, i32, i32, vp]),
            "eet_op_linear_strided": (i32, [vp, i64, vp, vp, vp, vp, i64, i64, i32, i32, i32, vp]),
            "eet_op_attention_prefill": (i32, [vp, vp, vp, vp, i32p, i32, i32, i32, i32, i32, vp]),
            "eet_op_attention_encoder": (i32, [vp, vp, vp, vp, i32p, i32, i32, i32, i32, i32, vp]),
            "eet_op_attention_unfused": (i32, [vp, vp, vp, vp, i32p, i32, i32, i32, i32, i32, vp, i32, vp]),
            "eet_op_attention_decode_scratch_bytes": (sz, [i32, i32, i32, i32]),
            "eet_op_attention_decode": (i32, [vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp]),
            "eet_op_attention_decode_static": (i32, [vp, vp, vp, vp, vp, i32, i32, i32, i32, vp]),
            "eet_model_workspace_bytes": (sz, [cfgp, C.POINTER(ModelConfig)]),
            "eet_model_create": (i32, [vp, cfgp, C.POINTER(ModelConfig), C.POINTER(ModelWeights), vp, C.POINTER(vp)]),
            "eet_model_prefill": (i32, [vp, i32p, i32, i32, vp, vp, vp, vp, vp]),
            "eet_model_prefill_left_padded": (i32, [vp, i32p, i32, i32, vp, vp, vp, vp, vp]),
            "eet_model_decode_step": (i32, [vp, vp, vp, vp, vp, vp]),
            "eet_model_hidden_states": (i32, [vp, C.POINTER(vp), C.POINTER(vp)]),
            "eet_model_destroy": (i32, [vp]),
            "eet_op_embedding": (i32, [vp, i32p, i32, i32, i32, i32, i32, vp, vp, vp, vp]),
            "eet_op_embedding_left_padded": (i32, [vp, i32p, i32, i32, i32, i32, i32, vp, vp, vp, vp]),
            "eet_op_embedding_decode": (i32, [vp, vp, i32, i32, i32, i32, vp, vp, vp, vp]),
            "eet_op_argmax": (i32, [vp, i32, i32, i32, vp, vp]),
            "eet_bufmgr_create": (i32, [vp, sz, C.POINTER(vp)]),
            "eet_bufmgr_request": (i32, [vp, sz, i32, C.POINTER(vp)]),
            "eet_bufmgr_release": (i32, [vp, vp]),
            "eet_bufmgr_query": (i32, [vp, C.POINTER(BufMgrStats)]),
            "eet_bufmgr_destroy": (i32, [vp]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


EXPORTS = ("eet_kv_cache_bytes", "eet_workspace_bytes", "eet_layer_create", "eet_prefill", "eet_prefill_left_padded",
           "eet_op_softmax_maskfree_left_padded", "eet_layer_encode", "eet_decode_step",
           "eet_cache_lens", "eet_layer_destroy", "eet_last_error", "eet_stack_kv_cache_bytes",
           "eet_stack_workspace_bytes", "eet_stack_create", "eet_stack_prefill", "eet_stack_decode_step",
           "eet_stack_cache_lens", "eet_stack_destroy", "eet_op_layernorm", "eet_op_softmax_maskfree",
           "eet_op_bias_gelu", "eet_op_bias_residual", "eet_op_linear", "eet_op_linear_strided", "eet_op_attention_prefill", "eet_op_attention_encoder",
           "eet_op_attention_unfused", "eet_op_attention_decode_scratch_bytes", "eet_op_attention_decode", "eet_op_attention_decode_static", "eet_bufmgr_create", "eet_bufmgr_request",
           "eet_bufmgr_release", "eet_bufmgr_query", "eet_bufmgr_destroy", "eet_model_workspace_bytes", "eet_model_create",
           "eet_model_prefill", "eet_model_decode_step", "eet_model_hidden_states", "eet_model_destroy", "eet_op_embedding",
           "eet_op_embedding_decode", "eet_op_argmax", "eet_stack_prefill_left_padded", "eet_model_prefill_left_padded",
           "eet_op_embedding_left_padded", "eet_stack_encode", "eet_restore", "eet_stack_restore")


def _check(code: int) -> None:
    if code != EET_OK:
        raise EETError(code, lib().eet_last_error().decode())


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_contiguous(), "tensors must be contiguous"
    return t.data_ptr()


def _stream(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def _lens_array(q_lens: Sequence[int]):
    return (C.c_int32 * len(q_lens))(*[int(v) for v in q_lens])


def make_config(hidden, heads, ffn, max_batch, max_prompt, max_seq, ln_eps=1e-5) -> LayerConfig:
    return LayerConfig(hidden, heads, ffn, max_batch, max_prompt, max_seq, ln_eps)


# ---- C ABI, same names --------------------------------------------------------------------
def eet_kv_cache_bytes(cfg: LayerConfig) -> int:
    return lib().eet_kv_cache_bytes(C.byref(cfg))


def eet_workspace_bytes(cfg: LayerConfig) -> int:
    return lib().eet_workspace_bytes(C.byref(cfg))


def eet_layer_create(cfg: LayerConfig, weights: Dict[str, torch.Tensor], workspace: torch.Tensor) -> int:
    w = LayerWeights(*[_ptr(weights[n]) for n in WEIGHT_FIELDS])
    handle = C.c_void_p()
    _check(lib().eet_layer_create(C.byref(cfg), C.byref(w), _ptr(workspace), C.byref(handle)))
    return handle.value


def eet_prefill(layer: int, q_lens: Sequence[int], batch: int, padded_len: int, tokens: torch.Tensor,
                out: torch.Tensor, kv_cache: torch.Tensor, stream=None) -> None:
    _check(lib().eet_prefill(layer, _lens_array(q_lens), batch, padded_len, _ptr(tokens), _ptr(out),
                             _ptr(kv_cache), _stream(stream)))


def eet_prefill_left_padded(layer: int, q_lens: Sequence[int], batch: int, padded_len: int, tokens: torch.Tensor,
                            out: torch.Tensor, kv_cache: torch.Tensor, stream=None) -> None:
    _check(lib().eet_prefill_left_padded(layer, _lens_array(q_lens), batch, padded_len, _ptr(tokens), _ptr(out),
                                         _ptr(kv_cache), _stream(stream)))


def eet_layer_encode(layer: int, q_lens: Sequence[int], batch: int, padded_len: int, tokens: torch.Tensor,
                     out: torch.Tensor, kv_scratch: torch.Tensor, stream=None) -> None:
    _check(lib().eet_layer_encode(layer, _lens_array(q_lens), batch, padded_len, _ptr(tokens), _ptr(out),
                                  _ptr(kv_scratch), _stream(stream)))


def eet_decode_step(layer: int, tokens: torch.Tensor, out: torch.Tensor, kv_cache: torch.Tensor, stream=None) -> None:
    _check(lib().eet_decode_step(layer, _ptr(tokens), _ptr(out), _ptr(kv_cache), _stream(stream)))


def eet_cache_lens(layer: int, batch: int, stream=None):
    out = (C.c_int32 * batch)()
    _check(lib().eet_cache_lens(layer, out, _stream(stream)))
    return list(out)


def eet_restore(layer: int, cache_lens: Sequence[int], stream=None) -> None:
    _check(lib().eet_restore(layer, _lens_array(cache_lens), len(cache_lens), _stream(stream)))


def eet_stack_restore(stack: int, cache_lens: Sequence[int], stream=None) -> None:
    _check(lib().eet_stack_restore(stack, _lens_array(cache_lens), len(cache_lens), _stream(stream)))


def eet_layer_destroy(layer: int) -> None:
    _check(lib().eet_layer_destroy(layer))


def eet_stack_kv_cache_bytes(cfg: LayerConfig, n_layers: int) -> int:
    return lib().eet_stack_kv_cache_bytes(C.byref(cfg), n_layers)


def eet_stack_workspace_bytes(cfg: LayerConfig, n_layers: int) -> int:
    return lib().eet_stack_workspace_bytes(C.byref(cfg), n_layers)


def eet_stack_create(cfg: LayerConfig, weights: Sequence[Dict[str, torch.Tensor]], workspace: torch.Tensor,
                     use_graph: bool = True) -> int:
    arr = (LayerWeights * len(weights))(*[LayerWeights(*[_ptr(w[n]) for n in WEIGHT_FIELDS]) for w in weights])
    handle = C.c_void_p()
    _check(lib().eet_stack_create(C.byref(cfg), len(weights), arr, _ptr(workspace), int(use_graph), C.byref(handle)))
    return handle.value


def eet_stack_prefill(stack: int, q_lens: Sequence[int], batch: int, padded_len: int, tokens, out, kv_cache,
                      stream=None) -> None:
    _check(lib().eet_stack_prefill(stack, _lens_array(q_lens), batch, padded_len, _ptr(tokens), _ptr(out),
                                   _ptr(kv_cache), _stream(stream)))


def eet_stack_prefill_left_padded(stack: int, q_lens: Sequence[int], batch: int, padded_len: int, tokens, out, kv_cache,
                                  stream=None) -> None:
    _check(lib().eet_stack_prefill_left_padded(stack, _lens_array(q_lens), batch, padded_len, _ptr(tokens), _ptr(out),
                                               _ptr(kv_cache), _stream(stream)))


def eet_stack_encode(stack: int, q_lens: Sequence[int], batch: int, padded_len: int, tokens, out, kv_scratch, stream=None) -> None:
    _check(lib().eet_stack_encode(stack, _lens_array(q_lens), batch, padded_len, _ptr(tokens), _ptr(out), _ptr(kv_scratch),
                                  _stream(stream)))


def eet_stack_decode_step(stack: int, tokens, out, kv_cache, stream=None) -> None:
    _check(lib().eet_stack_decode_step(stack, _ptr(tokens), _ptr(out), _ptr(kv_cache), _stream(stream)))


def eet_stack_cache_lens(stack: int, batch: int, stream=None):
    out = (C.c_int32 * batch)()
    _check(lib().eet_stack_cache_lens(stack, out, _stream(stream)))
    return list(out)


def eet_stack_destroy(stack: int) -> None:
    _check(lib().eet_stack_destroy(stack))


def eet_op_layernorm(x, gamma, beta, y, eps=1e-5, stream=None) -> None:
    rows, width = x.numel() // x.shape[-1], x.shape[-1]
    _check(lib().eet_op_layernorm(_ptr(x), _ptr(gamma), _ptr(beta), _ptr(y), rows, width, eps, _stream(stream)))


def eet_op_softmax_maskfree(scores, q_lens, scale=1.0, stream=None) -> None:
    B, nh, S, S2 = scores.shape
    assert S == S2
    _check(lib().eet_op_softmax_maskfree(_ptr(scores), _lens_array(q_lens), B, nh, S, scale, _stream(stream)))


def eet_op_softmax_maskfree_left_padded(scores, q_lens, scale=1.0, stream=None) -> None:
    B, nh, S, S2 = scores.shape
    assert S == S2
    _check(lib().eet_op_softmax_maskfree_left_padded(_ptr(scores), _lens_array(q_lens), B, nh, S, scale, _stream(stream)))


def eet_op_bias_gelu(x, bias, y, stream=None) -> None:
    _check(lib().eet_op_bias_gelu(_ptr(x), _ptr(bias), _ptr(y), x.numel() // x.shape[-1], x.shape[-1], _stream(stream)))


def eet_op_bias_residual(x, bias, residual, y, stream=None) -> None:
    _check(lib().eet_op_bias_residual(_ptr(x), _ptr(bias), _ptr(residual), _ptr(y), x.numel() // x.shape[-1],
                                      x.shape[-1], _stream(stream)))


def eet_op_linear(x, w, bias, y, residual=None, act=0, stream=None) -> None:
    rows, k = x.numel() // x.shape[-1], x.shape[-1]
    assert w.shape[1] == k
    _check(lib().eet_op_linear(_ptr(x), _ptr(w), _ptr(bias), _ptr(residual), _ptr(y), rows, k, w.shape[0], act,
                               _stream(stream)))


def eet_op_linear_strided(x, w, bias, y, residual=None, act=0, stream=None) -> None:
    """x [rows, in] and y [rows, out] may be column slices of wider contiguous buffers: their row strides are passed on."""
    assert x.dim() == 2 and y.dim() == 2 and x.stride(1) == 1 and y.stride(1) == 1 and x.shape[0] == y.shape[0]
    rows, k = x.shape
    assert w.shape[1] == k and y.shape[1] == w.shape[0]
    _check(lib().eet_op_linear_strided(x.data_ptr(), x.stride(0), _ptr(w), _ptr(bias), _ptr(residual), y.data_ptr(), y.stride(0),
                                       rows, k, w.shape[0], act, _stream(stream)))


def eet_op_attention_prefill(q, k_cache, v_cache, ctx, q_lens, heads, stream=None) -> None:
    B, S, H = q.shape
    _, nh, cap, d = k_cache.shape
    assert nh == heads and nh * d == H
    _check(lib().eet_op_attention_prefill(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(ctx), _lens_array(q_lens),
                                          B, S, heads, d, cap, _stream(stream)))


def eet_op_attention_encoder(q, k_cache, v_cache, ctx, q_lens, heads, stream=None) -> None:
    B, S, H = q.shape
    _, nh, cap, d = k_cache.shape
    assert nh == heads and nh * d == H
    _check(lib().eet_op_attention_encoder(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(ctx), _lens_array(q_lens),
                                          B, S, heads, d, cap, _stream(stream)))


def eet_op_attention_unfused(q, k_cache, v_cache, ctx, q_lens, heads, buffers, module: int = 0, stream=None) -> None:
    B, S, H = q.shape
    _, nh, cap, d = k_cache.shape
    assert nh == heads and nh * d == H
    _check(lib().eet_op_attention_unfused(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(ctx), _lens_array(q_lens),
                                          B, S, heads, d, cap, buffers, module, _stream(stream)))


def eet_op_attention_decode_scratch_bytes(batch, heads, d, capacity) -> int:
    return lib().eet_op_attention_decode_scratch_bytes(batch, heads, d, capacity)


def eet_op_attention_decode(q, k_cache, v_cache, ctx, n_keys, scratch, stream=None) -> None:
    B, nh, cap, d = k_cache.shape
    assert n_keys.dtype == torch.int32 and n_keys.is_cuda
    _check(lib().eet_op_attention_decode(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(ctx), _ptr(n_keys), B, nh, d,
                                         cap, _ptr(scratch), _stream(stream)))


def eet_op_attention_decode_static(q, k_cache, v_cache, ctx, n_keys, stream=None) -> None:
    B, nh, cap, d = k_cache.shape
    assert n_keys.dtype == torch.int32 and n_keys.is_cuda
    _check(lib().eet_op_attention_decode_static(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(ctx), _ptr(n_keys), B, nh, d,
                                                cap, _stream(stream)))


def eet_op_embedding(ids, q_lens, wte, wpe, out, vocab: Optional[int] = None, stream=None) -> None:
    B, S = ids.shape
    assert ids.dtype == torch.int32 and ids.is_cuda
    _check(lib().eet_op_embedding(_ptr(ids), _lens_array(q_lens), B, S, wte.shape[1], wte.shape[0] if vocab is None else vocab,
                                  wpe.shape[0], _ptr(wte), _ptr(wpe), _ptr(out), _stream(stream)))


def eet_op_embedding_left_padded(ids, q_lens, wte, wpe, out, vocab: Optional[int] = None, stream=None) -> None:
    B, S = ids.shape
    assert ids.dtype == torch.int32 and ids.is_cuda
    _check(lib().eet_op_embedding_left_padded(_ptr(ids), _lens_array(q_lens), B, S, wte.shape[1],
                                              wte.shape[0] if vocab is None else vocab, wpe.shape[0], _ptr(wte), _ptr(wpe),
                                              _ptr(out), _stream(stream)))


def eet_op_embedding_decode(ids, positions, wte, wpe, out, vocab: Optional[int] = None, stream=None) -> None:
    assert ids.dtype == torch.int32 and positions.dtype == torch.int32 and ids.is_cuda and positions.is_cuda
    _check(lib().eet_op_embedding_decode(_ptr(ids), _ptr(positions), ids.shape[0], wte.shape[1],
                                         wte.shape[0] if vocab is None else vocab, wpe.shape[0], _ptr(wte), _ptr(wpe), _ptr(out),
                                         _stream(stream)))


def eet_op_argmax(logits, out, vocab: Optional[int] = None, stream=None) -> None:
    rows, stride = logits.shape
    assert out.dtype == torch.int32 and out.is_cuda
    _check(lib().eet_op_argmax(_ptr(logits), rows, stride if vocab is None else vocab, stride, _ptr(out), _stream(stream)))


def eet_model_workspace_bytes(cfg: LayerConfig, mcfg: ModelConfig) -> int:
    return lib().eet_model_workspace_bytes(C.byref(cfg), C.byref(mcfg))


def eet_model_create(stack: int, cfg: LayerConfig, mcfg: ModelConfig, weights: Dict[str, torch.Tensor], workspace) -> int:
    w = ModelWeights(*[_ptr(weights[n]) for n in MODEL_WEIGHT_FIELDS])
    handle = C.c_void_p()
    _check(lib().eet_model_create(stack, C.byref(cfg), C.byref(mcfg), C.byref(w), _ptr(workspace), C.byref(handle)))
    return handle.value


def eet_model_prefill(model: int, q_lens: Sequence[int], batch: int, padded_len: int, ids, logits, next_ids, kv_cache,
                      stream=None) -> None:
    _check(lib().eet_model_prefill(model, _lens_array(q_lens), batch, padded_len, _ptr(ids), _ptr(logits), _ptr(next_ids),
                                   _ptr(kv_cache), _stream(stream)))


def eet_model_prefill_left_padded(model: int, q_lens: Sequence[int], batch: int, padded_len: int, ids, logits, next_ids,
                                  kv_cache, stream=None) -> None:
    _check(lib().eet_model_prefill_left_padded(model, _lens_array(q_lens), batch, padded_len, _ptr(ids), _ptr(logits),
                                               _ptr(next_ids), _ptr(kv_cache), _stream(stream)))


def eet_model_decode_step(model: int, ids, logits, next_ids, kv_cache, stream=None) -> None:
    _check(lib().eet_model_decode_step(model, _ptr(ids), _ptr(logits), _ptr(next_ids), _ptr(kv_cache), _stream(stream)))


def eet_model_hidden_states(model: int):
    """Device addresses (ints) of the input of layer 0 and the output of the last layer of the latest call."""
    a, b = C.c_void_p(), C.c_void_p()
    _check(lib().eet_model_hidden_states(model, C.byref(a), C.byref(b)))
    return a.value, b.value


def eet_model_destroy(model: int) -> None:
    _check(lib().eet_model_destroy(model))


# ---- convenience holder: allocates workspace and cache with torch, keeps tensors alive -------------
def eet_bufmgr_create(arena_ptr: int, arena_bytes: int) -> C.c_void_p:
    """arena_ptr: address of caller-owned device memory (an int: the manager never dereferences it)."""
    h = C.c_void_p()
    _check(lib().eet_bufmgr_create(arena_ptr, arena_bytes, C.byref(h)))
    return h


def eet_bufmgr_request(handle, nbytes: int, module: int) -> int:
    p = C.c_void_p()
    _check(lib().eet_bufmgr_request(handle, nbytes, module, C.byref(p)))
    return p.value


def eet_bufmgr_release(handle, buffer_ptr: int) -> None:
    _check(lib().eet_bufmgr_release(handle, buffer_ptr))


def eet_bufmgr_query(handle) -> BufMgrStats:
    st = BufMgrStats()
    _check(lib().eet_bufmgr_query(handle, C.byref(st)))
    return st


def eet_bufmgr_destroy(handle) -> None:
    _check(lib().eet_bufmgr_destroy(handle))


def _buffers_ready() -> None:
    """The holders below fill the K/V cache and upload the weights on torch's current stream, and their calls accept
    any stream: the library orders nothing across streams (include/eet.h), so the holder waits here, once, until what
    it allocated is in place."""
    torch.cuda.current_stream().synchronize()


class DecoderLayer:
    """Owns the torch buffers a layer handle borrows.  No arithmetic here."""

    def __init__(self, cfg: LayerConfig, weights: Dict[str, torch.Tensor], device="cuda:0", cache_fill: float = 0.0):
        self.cfg = cfg
        self.weights = {n: weights[n].to(device=device, dtype=torch.float16).contiguous() for n in WEIGHT_FIELDS}
        self.workspace = torch.empty(eet_workspace_bytes(cfg), dtype=torch.uint8, device=device)
        self.kv_cache = torch.full((eet_kv_cache_bytes(cfg) // 2,), cache_fill, dtype=torch.float16, device=device)
        self.handle = eet_layer_create(cfg, self.weights, self.workspace)
        _buffers_ready()

    def cache_views(self):
        c = self.cfg
        kv = self.kv_cache.view(2, c.max_batch, c.heads, c.max_seq, c.hidden // c.heads)
        return kv[0], kv[1]

    def prefill(self, tokens: torch.Tensor, q_lens: Sequence[int], out: Optional[torch.Tensor] = None, stream=None):
        B, S, _ = tokens.shape
        out = torch.empty_like(tokens) if out is None else out
        eet_prefill(self.handle, q_lens, B, S, tokens, out, self.kv_cache, stream)
        return out

    def prefill_left_padded(self, tokens: torch.Tensor, q_lens: Sequence[int], out: Optional[torch.Tensor] = None, stream=None):
        B, S, _ = tokens.shape
        out = torch.empty_like(tokens) if out is None else out
        eet_prefill_left_padded(self.handle, q_lens, B, S, tokens, out, self.kv_cache, stream)
        return out

    def encode(self, tokens: torch.Tensor, q_lens: Sequence[int], out: Optional[torch.Tensor] = None, stream=None):
        B, S, _ = tokens.shape
        out = torch.empty_like(tokens) if out is None else out
        eet_layer_encode(self.handle, q_lens, B, S, tokens, out, self.kv_cache, stream)
        return out

    def decode_step(self, tokens: torch.Tensor, out: Optional[torch.Tensor] = None, stream=None):
        out = torch.empty_like(tokens) if out is None else out
        eet_decode_step(self.handle, tokens, out, self.kv_cache, stream)
        return out

    def cache_lens(self, batch: int):
        return eet_cache_lens(self.handle, batch)

    def close(self):
        if self.handle:
            eet_layer_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class DecoderStack:
    """Owns the torch buffers a stack handle borrows (weights, workspace, K/V caches of all layers)."""

    def __init__(self, cfg: LayerConfig, weights: Sequence[Dict[str, torch.Tensor]], device="cuda:0",
                 cache_fill: float = 0.0, use_graph: bool = True):
        self.cfg, self.n_layers = cfg, len(weights)
        self.weights = [{n: w[n].to(device=device, dtype=torch.float16).contiguous() for n in WEIGHT_FIELDS}
                        for w in weights]
        self.workspace = torch.empty(eet_stack_workspace_bytes(cfg, self.n_layers), dtype=torch.uint8, device=device)
        self.kv_cache = torch.full((eet_stack_kv_cache_bytes(cfg, self.n_layers) // 2,), cache_fill,
                                   dtype=torch.float16, device=device)
        self.handle = eet_stack_create(cfg, self.weights, self.workspace, use_graph)
        _buffers_ready()

    def cache_views(self, layer: int):
        c = self.cfg
        kv = self.kv_cache.view(self.n_layers, 2, c.max_batch, c.heads, c.max_seq, c.hidden // c.heads)
        return kv[layer, 0], kv[layer, 1]

    def prefill(self, tokens: torch.Tensor, q_lens: Sequence[int], out: Optional[torch.Tensor] = None, stream=None):
        B, S, _ = tokens.shape
        out = torch.empty_like(tokens) if out is None else out
        eet_stack_prefill(self.handle, q_lens, B, S, tokens, out, self.kv_cache, stream)
        return out

    def prefill_left_padded(self, tokens: torch.Tensor, q_lens: Sequence[int], out: Optional[torch.Tensor] = None, stream=None):
        B, S, _ = tokens.shape
        out = torch.empty_like(tokens) if out is None else out
        eet_stack_prefill_left_padded(self.handle, q_lens, B, S, tokens, out, self.kv_cache, stream)
        return out

    def encode(self, tokens: torch.Tensor, q_lens: Sequence[int], out: Optional[torch.Tensor] = None, stream=None):
        """All layers as a bidirectional encoder; the first layer's share of the K/V cache serves as the scratch."""
        B, S, _ = tokens.shape
        out = torch.empty_like(tokens) if out is None else out
        eet_stack_encode(self.handle, q_lens, B, S, tokens, out, self.kv_cache, stream)
        return out

    def decode_step(self, tokens: torch.Tensor, out: Optional[torch.Tensor] = None, stream=None):
        out = torch.empty_like(tokens) if out is None else out
        eet_stack_decode_step(self.handle, tokens, out, self.kv_cache, stream)
        return out

    def cache_lens(self, batch: int):
        return eet_stack_cache_lens(self.handle, batch)

    def close(self):
        if self.handle:
            eet_stack_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class DecoderModel:
    """A DecoderStack plus the embedding tables and the final LayerNorm: token ids in, logits and greedy tokens out.
    Owns the torch buffers the model handle borrows.  No arithmetic here."""

    def __init__(self, cfg: LayerConfig, layer_weights: Sequence[Dict[str, torch.Tensor]], head: Dict[str, torch.Tensor],
                 vocab: int, device="cuda:0", cache_fill: float = 0.0, use_graph: bool = True):
        self.stack = DecoderStack(cfg, layer_weights, device=device, cache_fill=cache_fill, use_graph=use_graph)
        self.cfg, self.vocab = cfg, vocab
        self.head = {n: head[n].to(device=device, dtype=torch.float16).contiguous() for n in MODEL_WEIGHT_FIELDS}
        vp = (vocab + 63) // 64 * 64
        if self.head["wte"].shape[0] < vp:          # rows up to the padded vocabulary exist in memory (zeros)
            pad = torch.zeros((vp - self.head["wte"].shape[0], cfg.hidden), dtype=torch.float16, device=device)
            self.head["wte"] = torch.cat([self.head["wte"], pad]).contiguous()
        self.mcfg = ModelConfig(vocab, vp, self.head["wpe"].shape[0])
        self.workspace = torch.empty(eet_model_workspace_bytes(cfg, self.mcfg), dtype=torch.uint8, device=device)
        self.handle = eet_model_create(self.stack.handle, cfg, self.mcfg, self.head, self.workspace)
        _buffers_ready()
        self.batch = 0

    def prefill(self, ids: torch.Tensor, q_lens: Sequence[int], stream=None, left_padded: bool = False):
        B, S = ids.shape
        logits = torch.empty((B, self.mcfg.vocab_padded), dtype=torch.float16, device=ids.device)
        nxt = torch.empty((B,), dtype=torch.int32, device=ids.device)
        (eet_model_prefill_left_padded if left_padded else eet_model_prefill)(
            self.handle, q_lens, B, S, ids, logits, nxt, self.stack.kv_cache, stream)
        self.batch, self.padded_len = B, S
        return logits, nxt

    def decode_step(self, ids: torch.Tensor, stream=None):
        logits = torch.empty((ids.shape[0], self.mcfg.vocab_padded), dtype=torch.float16, device=ids.device)
        nxt = torch.empty((ids.shape[0],), dtype=torch.int32, device=ids.device)
        eet_model_decode_step(self.handle, ids, logits, nxt, self.stack.kv_cache, stream)
        return logits, nxt

    def hidden_states(self, decode: bool):
        """Views of the activation caches after the latest call: (input of layer 0, output of the last layer)."""
        shape = (self.batch, self.cfg.hidden) if decode else (self.batch, self.padded_len, self.cfg.hidden)
        n = 2 * self.batch * self.cfg.hidden * (1 if decode else self.padded_len)
        out = []
        for addr in eet_model_hidden_states(self.handle):
            view = None
            for buf in (self.stack.workspace, self.workspace):
                off = -1 if addr is None else addr - buf.data_ptr()
                if 0 <= off and off + n <= buf.numel():
                    view = buf[off: off + n].view(torch.float16).view(shape)
            out.append(view)                        # None: the buffer has been reused (see eet_model_hidden_states)
        assert out[1] is not None
        return out[0], out[1]

    def close(self):
        if self.handle:
            eet_model_destroy(self.handle)
            self.handle = None
        self.stack.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
