"""ctypes binding of libdash_attn.so: argument marshalling only.

Every function mirrors one entry point of include/dash_attn.h and takes torch
tensors that already live on the GPU; torch is used for device memory and the
current stream, nothing else.  There is no fallback: if the library is missing
or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import math
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("DASH_ATTN_LIB") or os.path.join(_HERE, "libdash_attn.so")

DASH_F32, DASH_BF16 = 0, 1


class DashError(RuntimeError):
    pass


class dash_params(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("h_q", ctypes.c_int32), ("h_kv", ctypes.c_int32),
        ("n_q", ctypes.c_int32), ("n_kv", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("block_size", ctypes.c_int32), ("causal", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("alpha", ctypes.c_float), ("gamma", ctypes.c_float), ("sigma", ctypes.c_float),
        ("scale", ctypes.c_float), ("window", ctypes.c_int32),
        ("q_stride", ctypes.c_int64 * 3), ("k_stride", ctypes.c_int64 * 3),
        ("v_stride", ctypes.c_int64 * 3), ("o_stride", ctypes.c_int64 * 3),
    ]


_lib = None
_P = ctypes.POINTER(dash_params)
_V = ctypes.c_void_p
_SIGNATURES = {
    "dash_list_stride": (ctypes.c_int32, [_P]),
    "dash_mask_words": (ctypes.c_int32, [_P]),
    "dash_attn_workspace_bytes": (ctypes.c_int, [_P, ctypes.POINTER(ctypes.c_size_t)]),
    "dash_kbar_compress": (ctypes.c_int, [_P, _V, _V, ctypes.c_int32, ctypes.c_int32, _V]),
    "dash_kbar_summarize": (ctypes.c_int, [_P, _V, _V, ctypes.POINTER(ctypes.c_int64), _V, ctypes.c_int32,
                                           ctypes.c_int32, _V]),
    "dash_stage1_route": (ctypes.c_int, [_P, _V, _V, _V, _V, _V, _V, _V, _V, ctypes.c_size_t, _V]),
    "dash_stage2_attend": (ctypes.c_int, [_P, _V, _V, _V, _V, _V, _V, _V, ctypes.c_size_t, _V]),
    "dash_attn_prefill": (ctypes.c_int, [_P, _V, _V, _V, _V, _V, _V, _V, _V, _V, _V, _V, ctypes.c_size_t, _V]),
    "dash_attn_decode": (ctypes.c_int, [_P, _V, _V, _V, _V, _V, _V, _V, _V, _V, _V, _V, ctypes.c_size_t, _V]),
    "dash_attn_decode_static": (ctypes.c_int, [_P, _V, _V, _V, _V, _V, _V, _V, _V, _V, _V, _V]),
    "dash_attn_decode_ragged": (ctypes.c_int, [_P, _V, _V, _V, _V, _V, ctypes.c_int32, _V, _V, _V, _V, _V, _V, _V,
                                               ctypes.c_size_t, _V]),
    "dense_attn": (ctypes.c_int, [_P, _V, _V, _V, _V, _V, ctypes.c_size_t, _V]),
    "dash_attn_backward_workspace_bytes": (ctypes.c_int, [_P, ctypes.POINTER(ctypes.c_size_t)]),
    "dash_attn_backward": (ctypes.c_int, [_P] + [_V] * 13 + [ctypes.c_size_t, _V]),
    "dash_kbar_summarize_backward": (ctypes.c_int, [_P, _V, _V, ctypes.POINTER(ctypes.c_int64), _V, _V, _V, _V]),
    "dash_strerror": (ctypes.c_char_p, [ctypes.c_int]),
}


def load_library(path: Optional[str] = None):
    """Load libdash_attn.so (built in-tree by paper_2605_18753_amd.build)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise DashError(f"{p} not found: build it with `python -m paper_2605_18753_amd.build`")
    lib = ctypes.CDLL(p)
    for name, (res, args) in _SIGNATURES.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    if path is None:
        _lib = lib
    return lib


def exported_symbols():
    return list(_SIGNATURES)


def _check(rc: int, what: str):
    if rc != 0:
        msg = load_library().dash_strerror(rc).decode()
        raise DashError(f"{what} failed: {msg} ({rc})")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_params(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, o: Optional[torch.Tensor],
                block: int, alpha: float = 1.5, gamma: float = 1.0, sigma: float = 1.0,
                causal: bool = True, scale: float = 0.0, window: int = 0) -> dash_params:
    """q [B,H_q,n_q,d]; k, v [B,H_kv,n_kv,d]; last dim contiguous."""
    p = dash_params()
    p.batch, p.h_q, p.n_q, p.head_dim = q.shape
    p.h_kv, p.n_kv = k.shape[1], k.shape[2]
    p.block_size = block
    p.causal = int(causal)
    p.dtype = DASH_BF16 if q.dtype == torch.bfloat16 else DASH_F32
    p.alpha, p.gamma, p.sigma, p.scale = alpha, gamma, sigma, scale
    p.window = window
    for name, t in (("q_stride", q), ("k_stride", k), ("v_stride", v), ("o_stride", o if o is not None else q)):
        assert t.stride(3) == 1, "head_dim must be contiguous"
        getattr(p, name)[:] = [t.stride(0), t.stride(1), t.stride(2)]
    return p


def workspace_bytes(p: dash_params) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().dash_attn_workspace_bytes(ctypes.byref(p), ctypes.byref(n)), "dash_attn_workspace_bytes")
    return n.value


def list_stride(p: dash_params) -> int:
    return load_library().dash_list_stride(ctypes.byref(p))


def mask_words(p: dash_params) -> int:
    return load_library().dash_mask_words(ctypes.byref(p))


def alloc_workspace(p: dash_params, device) -> torch.Tensor:
    return torch.empty(workspace_bytes(p) + 256, dtype=torch.uint8, device=device)


def _ws_ptr(ws: torch.Tensor):
    base = ws.data_ptr()
    aligned = (base + 255) & ~255
    return ctypes.c_void_p(aligned), ws.numel() - (aligned - base)


@dataclass
class Lists:
    """Optional Stage-1 outputs (see dash_stage1_route in the header)."""
    mask: Optional[torch.Tensor] = None
    cnt: Optional[torch.Tensor] = None
    idx: Optional[torch.Tensor] = None
    bias: Optional[torch.Tensor] = None
    tau: Optional[torch.Tensor] = None

    @staticmethod
    def allocate(p: dash_params, device, idx: bool = True, tau: bool = True) -> "Lists":
        rows = (p.batch, p.h_kv, p.n_q)
        ls, mw = list_stride(p), mask_words(p)
        return Lists(
            mask=torch.zeros(rows + (mw,), dtype=torch.int32, device=device),
            cnt=torch.zeros(rows, dtype=torch.int32, device=device),
            idx=torch.zeros(rows + (ls,), dtype=torch.int32, device=device) if idx else None,
            bias=torch.zeros(rows + (ls,), dtype=torch.float32, device=device),
            tau=torch.zeros((p.batch, p.h_q, p.n_q), dtype=torch.float32, device=device) if tau else None,
        )


def dash_kbar_compress(p: dash_params, k: torch.Tensor, kbar: torch.Tensor,
                       first_chunk: int = 0, n_chunks: int = -1) -> None:
    _check(load_library().dash_kbar_compress(ctypes.byref(p), _ptr(k), _ptr(kbar), first_chunk, n_chunks,
                                             _stream()), "dash_kbar_compress")


def _qbar_strides(qbar: torch.Tensor):
    assert qbar.dtype == torch.float32 and qbar.stride(-1) == 1
    if qbar.dim() == 2:
        st = (0, qbar.stride(0), 0)
    elif qbar.dim() == 3:
        st = (0, qbar.stride(0), qbar.stride(1))
    else:
        st = (qbar.stride(0), qbar.stride(1), qbar.stride(2))
    return (ctypes.c_int64 * 3)(*st)


def dash_kbar_summarize(p: dash_params, k: torch.Tensor, qbar: torch.Tensor, kbar: torch.Tensor,
                        first_chunk: int = 0, n_chunks: int = -1) -> None:
    """qbar: fp32 tensor [h_kv, d] (one summary query per kv-head), [h_kv, T_c, d]
    or [batch, h_kv, T_c, d] (one per chunk); only the strides are passed on."""
    arr = _qbar_strides(qbar)
    _check(load_library().dash_kbar_summarize(ctypes.byref(p), _ptr(k), _ptr(qbar), arr, _ptr(kbar),
                                              first_chunk, n_chunks, _stream()), "dash_kbar_summarize")


def dash_stage1_route(p, q, kbar, lists: Lists, ws: torch.Tensor) -> None:
    wp, wn = _ws_ptr(ws)
    _check(load_library().dash_stage1_route(ctypes.byref(p), _ptr(q), _ptr(kbar), _ptr(lists.mask),
                                            _ptr(lists.cnt), _ptr(lists.idx), _ptr(lists.bias),
                                            _ptr(lists.tau), wp, wn, _stream()), "dash_stage1_route")


def dash_stage2_attend(p, q, k, v, o, lists: Lists, ws: torch.Tensor) -> None:
    wp, wn = _ws_ptr(ws)
    _check(load_library().dash_stage2_attend(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(o),
                                             _ptr(lists.mask), _ptr(lists.bias), wp, wn, _stream()),
           "dash_stage2_attend")


def dash_attn_prefill(p, q, k, v, o, kbar, lists: Lists, ws: torch.Tensor) -> None:
    wp, wn = _ws_ptr(ws)
    _check(load_library().dash_attn_prefill(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(kbar),
                                            _ptr(lists.mask), _ptr(lists.cnt), _ptr(lists.idx),
                                            _ptr(lists.bias), _ptr(lists.tau), wp, wn, _stream()),
           "dash_attn_prefill")


def dash_attn_decode(p, q, k_cache, v_cache, kbar_cache, o, lists: Lists, ws: torch.Tensor) -> None:
    wp, wn = _ws_ptr(ws)
    _check(load_library().dash_attn_decode(ctypes.byref(p), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                           _ptr(kbar_cache), _ptr(o), _ptr(lists.mask), _ptr(lists.cnt),
                                           _ptr(lists.idx), _ptr(lists.bias), _ptr(lists.tau), wp, wn,
                                           _stream()), "dash_attn_decode")


def dash_attn_decode_static(p, q, k_cache, v_cache, kbar_cache, o, lists: Lists) -> None:
    """dash_attn_decode on the library's built-in scratch (no workspace, no allocation)."""
    _check(load_library().dash_attn_decode_static(ctypes.byref(p), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                                  _ptr(kbar_cache), _ptr(o), _ptr(lists.mask), _ptr(lists.cnt),
                                                  _ptr(lists.idx), _ptr(lists.bias), _ptr(lists.tau), _stream()),
           "dash_attn_decode_static")


def dash_attn_decode_ragged(p, q, k_cache, v_cache, kbar_cache, seq_lens: torch.Tensor, o, lists: Lists,
                            ws: torch.Tensor, update_cache: bool = True) -> None:
    assert seq_lens.dtype == torch.int32 and seq_lens.is_contiguous() and seq_lens.numel() == p.batch
    wp, wn = _ws_ptr(ws)
    _check(load_library().dash_attn_decode_ragged(ctypes.byref(p), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                                  _ptr(kbar_cache), _ptr(seq_lens), int(update_cache), _ptr(o),
                                                  _ptr(lists.mask), _ptr(lists.cnt), _ptr(lists.idx),
                                                  _ptr(lists.bias), _ptr(lists.tau), wp, wn, _stream()),
           "dash_attn_decode_ragged")


def dense_attn(p, q, k, v, o, ws: torch.Tensor) -> None:
    wp, wn = _ws_ptr(ws)
    _check(load_library().dense_attn(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(o), wp, wn, _stream()),
           "dense_attn")


def backward_workspace_bytes(p: dash_params) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().dash_attn_backward_workspace_bytes(ctypes.byref(p), ctypes.byref(n)),
           "dash_attn_backward_workspace_bytes")
    return n.value


def alloc_backward_workspace(p: dash_params, device) -> torch.Tensor:
    return torch.empty(backward_workspace_bytes(p) + 256, dtype=torch.uint8, device=device)


def dash_attn_backward(p, q, k, v, d_o, kbar, lists: Lists, dq, dk, dv, ws: torch.Tensor, dkbar=None) -> None:
    """Backward of dash_attn_prefill; lists.mask / bias / tau are the forward's outputs.
    dkbar None: block-mean summaries (their gradient is folded into dk)."""
    wp, wn = _ws_ptr(ws)
    if dkbar is not None:
        assert dkbar.dtype == torch.float32 and dkbar.is_contiguous() and tuple(dkbar.shape) == kbar_shape(p)
    _check(load_library().dash_attn_backward(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(d_o),
                                             _ptr(kbar), _ptr(lists.mask), _ptr(lists.bias), _ptr(lists.tau),
                                             _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dkbar), wp, wn, _stream()),
           "dash_attn_backward")


def dash_kbar_summarize_backward(p, k, qbar: torch.Tensor, dkbar: torch.Tensor, dk, dqbar: torch.Tensor) -> None:
    """Backward of dash_kbar_summarize; qbar as there ([h_kv,d], [h_kv,T_c,d] or [batch,h_kv,T_c,d])."""
    strides = _qbar_strides(qbar)
    assert dkbar.dtype == torch.float32 and dkbar.is_contiguous() and tuple(dkbar.shape) == kbar_shape(p)
    assert dqbar.dtype == torch.float32 and dqbar.is_contiguous() and tuple(dqbar.shape) == kbar_shape(p)
    _check(load_library().dash_kbar_summarize_backward(ctypes.byref(p), _ptr(k), _ptr(qbar), strides, _ptr(dkbar),
                                                       _ptr(dk), _ptr(dqbar), _stream()),
           "dash_kbar_summarize_backward")


def kbar_shape(p: dash_params):
    return (p.batch, p.h_kv, p.n_kv // p.block_size, p.head_dim)
