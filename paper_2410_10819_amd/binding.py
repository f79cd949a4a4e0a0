"""ctypes binding of libduoattn.so / libduosynth.so: argument marshalling only.

Function names and argument order follow include/duoattn.h.  Tensors are torch
CUDA tensors (PyTorch is used for device memory and streams, nothing else);
every step of the attention path runs inside the library's HIP kernels.  There
is no fallback: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("DUOATTN_LIB") or os.path.join(_HERE, "libduoattn.so")
SYNTH_LIB_PATH = os.path.join(_HERE, "libduosynth.so")

DUO_OK, DUO_EINVAL, DUO_ENOMEM, DUO_ERANGE, DUO_ESTATE, DUO_EHIP = 0, -1, -2, -3, -4, -5
DUO_KV_BF16, DUO_KV_FP8_E4M3, DUO_KV_INT4, DUO_KV_INT8 = 0, 1, 2, 3


class DuoError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("duoattn status %d: %s" % (status, message))
        self.status = status
        self.message = message


class duo_config_t(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("sink", ctypes.c_int32),
                ("recent", ctypes.c_int32), ("max_seq", ctypes.c_int64), ("kv_dtype", ctypes.c_int32),
                ("retrieval_mask", ctypes.c_void_p), ("softmax_scale", ctypes.c_float)]


class duo_call_params_t(ctypes.Structure):
    _fields_ = [("head_mask", ctypes.c_void_p), ("sink", ctypes.c_int32), ("recent", ctypes.c_int32)]


_lib = None
_synth = None


def load() -> ctypes.CDLL:
    """Load libduoattn.so (built in-tree by build.py); raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("%s not found: run `python -m paper_2410_10819_amd.build` first" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    lib.duo_last_error.restype = ctypes.c_char_p
    lib.duo_last_error.argtypes = []
    lib.duo_cache_create.argtypes = [ctypes.POINTER(duo_config_t), ctypes.POINTER(vp)]
    lib.duo_cache_destroy.argtypes = [vp]
    lib.duo_cache_reset.argtypes = [vp]
    lib.duo_cache_len.argtypes = [vp, i32]
    lib.duo_cache_len.restype = i64
    lib.duo_cache_bytes.argtypes = [vp]
    lib.duo_cache_bytes.restype = i64
    lib.duo_set_decode_splits.argtypes = [vp, i32]
    lib.duo_set_decode_kernel.argtypes = [vp, i32]
    lib.duo_kv_append.argtypes = [vp, i32, vp, vp, i32, ctypes.POINTER(duo_call_params_t), vp]
    lib.duo_attn_prefill.argtypes = [vp, i32, vp, vp, vp, i32, ctypes.POINTER(duo_call_params_t), vp, vp, vp]
    lib.duo_attn_prefill_deployed.argtypes = lib.duo_attn_prefill.argtypes
    lib.duo_attn_gate_mixed.argtypes = [vp, i32, vp, vp, vp, i32, ctypes.POINTER(ctypes.c_float), i32, vp, vp, vp]
    lib.duo_attn_decode.argtypes = [vp, i32, vp, vp, vp, ctypes.POINTER(duo_call_params_t), vp, vp, vp]
    lib.duo_decode_step.argtypes = lib.duo_attn_decode.argtypes
    lib.duo_attn_decode_static.argtypes = lib.duo_attn_decode.argtypes
    lib.duo_cache_export.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp, i64, ctypes.POINTER(i64), vp]
    _lib = lib
    return lib


def load_synth() -> ctypes.CDLL:
    global _synth
    if _synth is None:
        if not os.path.exists(SYNTH_LIB_PATH):
            raise ImportError("%s not found: run `python -m paper_2410_10819_amd.build` first" % SYNTH_LIB_PATH)
        s = ctypes.CDLL(SYNTH_LIB_PATH)
        s.duo_synth_fill_bf16.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int64,
                                          ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
        _synth = s
    return _synth


def _check(status: int):
    if status != DUO_OK:
        raise DuoError(status, load().duo_last_error().decode())


def _ptr(t, name, dtype=None):
    """Device address of a contiguous torch CUDA tensor (None -> NULL)."""
    if t is None:
        return None
    if isinstance(t, int):          # a raw device address the caller already validated
        return ctypes.c_void_p(t)
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a torch CUDA tensor" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s must have dtype %s, got %s" % (name, dtype, t.dtype))
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    return ctypes.c_void_p(int(stream))


def _params(params):
    """params: None or (head_mask uint8 numpy [n_kv_heads] or None, sink, recent)."""
    if params is None:
        return None, None
    mask, sink, recent = params
    keep = None
    p = duo_call_params_t()
    if mask is not None:
        keep = np.ascontiguousarray(mask, dtype=np.uint8)
        p.head_mask = keep.ctypes.data
    p.sink, p.recent = int(sink), int(recent)
    return ctypes.byref(p), (p, keep)


def duo_cache_create(n_layers, batch, n_q_heads, n_kv_heads, head_dim, sink, recent, max_seq,
                     retrieval_mask, kv_dtype=DUO_KV_BF16, softmax_scale=0.0):
    """Returns the opaque handle (ctypes.c_void_p)."""
    lib = load()
    cfg = duo_config_t()
    cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads = n_layers, batch, n_q_heads, n_kv_heads
    cfg.head_dim, cfg.sink, cfg.recent, cfg.max_seq = head_dim, sink, recent, max_seq
    cfg.kv_dtype, cfg.softmax_scale = kv_dtype, softmax_scale
    mask = None
    if retrieval_mask is not None:
        mask = np.ascontiguousarray(retrieval_mask, dtype=np.uint8)
        if mask.size != max(n_layers, 0) * max(n_kv_heads, 0):
            raise ValueError("retrieval_mask must hold n_layers * n_kv_heads entries")
        cfg.retrieval_mask = mask.ctypes.data
    handle = ctypes.c_void_p()
    _check(lib.duo_cache_create(ctypes.byref(cfg), ctypes.byref(handle)))
    return handle


def duo_cache_destroy(cache):
    _check(load().duo_cache_destroy(cache))


def duo_cache_reset(cache):
    _check(load().duo_cache_reset(cache))


def duo_cache_len(cache, layer) -> int:
    n = load().duo_cache_len(cache, layer)
    if n < 0:
        _check(int(n))
    return int(n)


def duo_cache_bytes(cache) -> int:
    return int(load().duo_cache_bytes(cache))


def duo_set_decode_splits(cache, splits):
    _check(load().duo_set_decode_splits(cache, splits))


def duo_set_decode_kernel(cache, kernel):
    _check(load().duo_set_decode_kernel(cache, kernel))


def duo_kv_append(cache, layer, k, v, n_new, params=None, stream=None):
    import torch
    pp, keep = _params(params)
    _check(load().duo_kv_append(cache, layer, _ptr(k, "k", torch.bfloat16), _ptr(v, "v", torch.bfloat16),
                                n_new, pp, _stream(stream)))


def duo_attn_prefill(cache, layer, q, k, v, n_new, out, lse=None, params=None, stream=None):
    import torch
    pp, keep = _params(params)
    _check(load().duo_attn_prefill(cache, layer, _ptr(q, "q", torch.bfloat16), _ptr(k, "k", torch.bfloat16),
                                   _ptr(v, "v", torch.bfloat16), n_new, pp, _ptr(out, "out", torch.bfloat16),
                                   _ptr(lse, "lse", torch.float32), _stream(stream)))


def duo_attn_prefill_deployed(cache, layer, q, k, v, n_new, out, lse=None, params=None, stream=None):
    import torch
    pp, keep = _params(params)
    _check(load().duo_attn_prefill_deployed(cache, layer, _ptr(q, "q", torch.bfloat16), _ptr(k, "k", torch.bfloat16),
                                            _ptr(v, "v", torch.bfloat16), n_new, pp, _ptr(out, "out", torch.bfloat16),
                                            _ptr(lse, "lse", torch.float32), _stream(stream)))


def duo_attn_gate_mixed(cache, layer, q, k, v, n_tokens, alpha, out, workspace=None, block=0, stream=None):
    """alpha: host float32 values, one per KV head; workspace: unused (kept for the C signature), may be None."""
    import torch
    al = np.ascontiguousarray(np.asarray(alpha, dtype=np.float32))
    _check(load().duo_attn_gate_mixed(cache, layer, _ptr(q, "q", torch.bfloat16), _ptr(k, "k", torch.bfloat16),
                                      _ptr(v, "v", torch.bfloat16), n_tokens,
                                      al.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), block,
                                      _ptr(out, "out", torch.bfloat16), _ptr(workspace, "workspace", torch.bfloat16),
                                      _stream(stream)))


def duo_attn_decode(cache, layer, q, out, k=None, v=None, lse=None, params=None, stream=None):
    import torch
    pp, keep = _params(params)
    _check(load().duo_attn_decode(cache, layer, _ptr(q, "q", torch.bfloat16), _ptr(k, "k", torch.bfloat16),
                                  _ptr(v, "v", torch.bfloat16), pp, _ptr(out, "out", torch.bfloat16),
                                  _ptr(lse, "lse", torch.float32), _stream(stream)))


def duo_attn_decode_static(cache, layer, q, out, k=None, v=None, lse=None, params=None, stream=None):
    import torch
    pp, keep = _params(params)
    _check(load().duo_attn_decode_static(cache, layer, _ptr(q, "q", torch.bfloat16), _ptr(k, "k", torch.bfloat16),
                                         _ptr(v, "v", torch.bfloat16), pp, _ptr(out, "out", torch.bfloat16),
                                         _ptr(lse, "lse", torch.float32), _stream(stream)))


def duo_decode_step(cache, layer, q, k, v, out, lse=None, params=None, stream=None):
    import torch
    pp, keep = _params(params)
    _check(load().duo_decode_step(cache, layer, _ptr(q, "q", torch.bfloat16), _ptr(k, "k", torch.bfloat16),
                                  _ptr(v, "v", torch.bfloat16), pp, _ptr(out, "out", torch.bfloat16),
                                  _ptr(lse, "lse", torch.float32), _stream(stream)))


def duo_cache_export(cache, layer, batch_idx, kv_head, k_out, v_out, positions_out, capacity,
                     kscale_out=None, vscale_out=None, stream=None) -> int:
    """Returns the number of rows written."""
    import torch
    count = ctypes.c_int64(0)
    _check(load().duo_cache_export(cache, layer, batch_idx, kv_head, _ptr(k_out, "k_out"), _ptr(v_out, "v_out"),
                                   _ptr(kscale_out, "kscale_out", torch.float32),
                                   _ptr(vscale_out, "vscale_out", torch.float32),
                                   _ptr(positions_out, "positions_out", torch.int64), capacity,
                                   ctypes.byref(count), _stream(stream)))
    return int(count.value)


def duo_synth_fill_bf16(dst, table, key, pos_start, n_pos, n_heads, head_dim, stream=None):
    import torch
    rc = load_synth().duo_synth_fill_bf16(_ptr(dst, "dst", torch.bfloat16), _ptr(table, "table"), key, pos_start,
                                          n_pos, n_heads, head_dim, _stream(stream))
    if rc != 0:
        raise DuoError(rc, "duo_synth_fill_bf16 failed")
