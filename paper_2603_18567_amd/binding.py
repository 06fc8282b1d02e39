"""ctypes binding of libttt_attn.so: same names as include/ttt_attn.h, argument marshalling only.

Every step of the path runs in the HIP kernels; PyTorch supplies device memory and the stream.
There is no fallback: if the library has not been built the first call raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

from .build import LIB_PATH

TTT_OK, TTT_ERR_INVALID_ARG, TTT_ERR_UNSUPPORTED, TTT_ERR_WORKSPACE, TTT_ERR_HIP = 0, -1, -2, -3, -4
TTT_F32, TTT_BF16 = 0, 1
TTT_PASS_FWD, TTT_PASS_BWD, TTT_PASS_BWD_ACCUM = 0, 1, 2
TTT_MAX_STEPS = 32

EXPORTS = ("ttt_attn_workspace_bytes", "ttt_attn_fwd", "ttt_attn_bwd", "ttt_attn_last_error",
           "ttt_attn_profile_enable", "ttt_attn_profile_totals", "ttt_attn_fwd_docsteps", "ttt_attn_bwd_docsteps",
           "ttt_loss_bwd_inplace", "ttt_qkv_rope_fwd", "ttt_o_proj_fwd", "ttt_attn_fwd_static")
TTT_STATIC_MAX_TOKENS = 524288


class TttAttnParams(ctypes.Structure):
    _fields_ = [
        ("dtype", ctypes.c_int32), ("k", ctypes.c_int32),
        ("step_begin", ctypes.c_int32), ("step_end", ctypes.c_int32),
        ("total_tokens", ctypes.c_int32), ("n_docs", ctypes.c_int32),
        ("hq", ctypes.c_int32), ("hkv", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("softmax_scale", ctypes.c_float),
        ("q_stride_token", ctypes.c_int64), ("q_stride_head", ctypes.c_int64),
        ("kv_stride_token", ctypes.c_int64), ("kv_stride_head", ctypes.c_int64),
    ]


class TttAttnError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"ttt_attn error {code}: {msg}")
        self.code = code


_lib = None


def load_library():
    """Load the in-tree shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2603_18567_amd.build` "
                "(there is no CPU or PyTorch fallback for TTT attention)")
        lib = ctypes.CDLL(LIB_PATH)
        vp, pp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p)
        lib.ttt_attn_workspace_bytes.restype = ctypes.c_size_t
        lib.ttt_attn_workspace_bytes.argtypes = [ctypes.POINTER(TttAttnParams), ctypes.c_int]
        lib.ttt_attn_fwd.restype = ctypes.c_int
        lib.ttt_attn_fwd.argtypes = [ctypes.POINTER(TttAttnParams), pp, pp, pp, vp, vp, pp, pp,
                                     vp, ctypes.c_size_t, vp]
        lib.ttt_attn_fwd_static.restype = ctypes.c_int
        lib.ttt_attn_fwd_static.argtypes = [ctypes.POINTER(TttAttnParams), pp, pp, pp, vp, vp, pp, pp, vp]
        lib.ttt_attn_bwd.restype = ctypes.c_int
        lib.ttt_attn_bwd.argtypes = [ctypes.POINTER(TttAttnParams), pp, pp, pp, pp, pp, pp, vp, vp,
                                     pp, pp, pp, ctypes.c_int, vp, ctypes.c_size_t, vp]
        lib.ttt_attn_fwd_docsteps.restype = ctypes.c_int
        lib.ttt_attn_fwd_docsteps.argtypes = [ctypes.POINTER(TttAttnParams), vp, pp, pp, pp, vp, vp, pp, pp,
                                              vp, ctypes.c_size_t, vp]
        lib.ttt_attn_bwd_docsteps.restype = ctypes.c_int
        lib.ttt_attn_bwd_docsteps.argtypes = [ctypes.POINTER(TttAttnParams), vp, pp, pp, pp, pp, pp, pp, vp, vp,
                                              pp, pp, pp, vp, ctypes.c_size_t, vp]
        lib.ttt_attn_last_error.restype = ctypes.c_char_p
        lib.ttt_attn_last_error.argtypes = []
        lib.ttt_attn_profile_enable.restype = ctypes.c_int
        lib.ttt_attn_profile_enable.argtypes = [ctypes.c_int]
        lib.ttt_attn_profile_totals.restype = ctypes.c_int
        lib.ttt_attn_profile_totals.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_char_p),
                                                ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int32)]
        lib.ttt_loss_bwd_inplace.restype = ctypes.c_int
        lib.ttt_loss_bwd_inplace.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_int32, ctypes.c_int64,
                                             ctypes.c_int64, ctypes.c_int32, vp]
        lib.ttt_qkv_rope_fwd.restype = ctypes.c_int
        lib.ttt_qkv_rope_fwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                         ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                                         ctypes.c_int32, vp]
        lib.ttt_o_proj_fwd.restype = ctypes.c_int
        lib.ttt_o_proj_fwd.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64,
                                       ctypes.c_int64, ctypes.c_int32, vp]
        _lib = lib
    return _lib


def ttt_attn_last_error() -> str:
    return load_library().ttt_attn_last_error().decode()


def ttt_attn_profile_enable(on: bool) -> bool:
    return bool(load_library().ttt_attn_profile_enable(int(bool(on))))


def ttt_attn_profile_totals(capacity: int = 16) -> dict:
    """{kernel name: total milliseconds} of the launches recorded since the last query (waits)."""
    names = (ctypes.c_char_p * capacity)()
    ms = (ctypes.c_float * capacity)()
    cnt = (ctypes.c_int32 * capacity)()
    n = load_library().ttt_attn_profile_totals(capacity, names, ms, cnt)
    return {names[i].decode(): float(ms[i]) for i in range(n)}


def _ptr_array(tensors, k):
    arr = (ctypes.c_void_p * k)()
    for i in range(k):
        t = tensors[i] if tensors is not None and i < len(tensors) else None
        arr[i] = None if t is None else t.data_ptr()
    return arr


def make_params(q_like, kv_like, k, step_begin, step_end, cu_seqlens_host, softmax_scale) -> TttAttnParams:
    """Parameter block from one [T,hq,d] and one [T,hkv,d] tensor (shapes, strides, dtype)."""
    T, hq, d = q_like.shape
    hkv = kv_like.shape[1]
    assert q_like.stride(2) == 1 and kv_like.stride(2) == 1, "head_dim must be contiguous"
    dt = {torch.float32: TTT_F32, torch.bfloat16: TTT_BF16}[q_like.dtype]
    return TttAttnParams(dt, k, step_begin, step_end, T, len(cu_seqlens_host) - 1, hq, hkv, d,
                         float(softmax_scale), q_like.stride(0), q_like.stride(1),
                         kv_like.stride(0), kv_like.stride(1))


def ttt_attn_workspace_bytes(params: TttAttnParams, which_pass: int) -> int:
    lib = load_library()
    n = lib.ttt_attn_workspace_bytes(ctypes.byref(params), which_pass)
    if n == 0:
        raise TttAttnError(TTT_ERR_INVALID_ARG, ttt_attn_last_error())
    return int(n)


def _stream_ptr(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _cu_host_array(cu_seqlens_host):
    vals = [int(x) for x in cu_seqlens_host]
    return (ctypes.c_int32 * len(vals))(*vals)


def ttt_attn_fwd(params, q, k, v, cu_seqlens_dev, cu_seqlens_host, o, lse, workspace, stream=None):
    """q,k,v,o,lse: lists (length params.k; None where a step is not needed) of device tensors."""
    lib = load_library()
    K = params.k
    rc = lib.ttt_attn_fwd(ctypes.byref(params), _ptr_array(q, K), _ptr_array(k, K), _ptr_array(v, K),
                          ctypes.c_void_p(cu_seqlens_dev.data_ptr()), _cu_host_array(cu_seqlens_host),
                          _ptr_array(o, K), _ptr_array(lse, K),
                          ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                          _stream_ptr(stream))
    if rc != TTT_OK:
        raise TttAttnError(rc, ttt_attn_last_error())


def ttt_attn_fwd_static(params, q, k, v, cu_seqlens_dev, cu_seqlens_host, o, lse, stream=None):
    """ttt_attn_fwd without a workspace (the library's built-in scratch; at most TTT_STATIC_MAX_TOKENS tokens)."""
    lib = load_library()
    K = params.k
    rc = lib.ttt_attn_fwd_static(ctypes.byref(params), _ptr_array(q, K), _ptr_array(k, K), _ptr_array(v, K),
                                 ctypes.c_void_p(cu_seqlens_dev.data_ptr()), _cu_host_array(cu_seqlens_host),
                                 _ptr_array(o, K), _ptr_array(lse, K), _stream_ptr(stream))
    if rc != TTT_OK:
        raise TttAttnError(rc, ttt_attn_last_error())


def _doc_steps_array(doc_steps, n_docs):
    assert len(doc_steps) == n_docs
    return (ctypes.c_int32 * max(n_docs, 1))(*[int(x) for x in doc_steps])


def ttt_attn_fwd_docsteps(params, doc_steps, q, k, v, cu_seqlens_dev, cu_seqlens_host, o, lse, workspace, stream=None):
    """ttt_attn_fwd with a step count per document (host list of n_docs integers in 0..k)."""
    lib = load_library()
    K = params.k
    rc = lib.ttt_attn_fwd_docsteps(ctypes.byref(params), _doc_steps_array(doc_steps, params.n_docs),
                                   _ptr_array(q, K), _ptr_array(k, K), _ptr_array(v, K),
                                   ctypes.c_void_p(cu_seqlens_dev.data_ptr()), _cu_host_array(cu_seqlens_host),
                                   _ptr_array(o, K), _ptr_array(lse, K),
                                   ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                                   _stream_ptr(stream))
    if rc != TTT_OK:
        raise TttAttnError(rc, ttt_attn_last_error())


def ttt_attn_bwd_docsteps(params, doc_steps, q, k, v, o, lse, d_o, cu_seqlens_dev, cu_seqlens_host, dq, dk, dv,
                          workspace, stream=None):
    """ttt_attn_bwd (no carry mode) with a step count per document."""
    lib = load_library()
    K = params.k
    rc = lib.ttt_attn_bwd_docsteps(ctypes.byref(params), _doc_steps_array(doc_steps, params.n_docs),
                                   _ptr_array(q, K), _ptr_array(k, K), _ptr_array(v, K),
                                   _ptr_array(o, K), _ptr_array(lse, K), _ptr_array(d_o, K),
                                   ctypes.c_void_p(cu_seqlens_dev.data_ptr()), _cu_host_array(cu_seqlens_host),
                                   _ptr_array(dq, K), _ptr_array(dk, K), _ptr_array(dv, K),
                                   ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                                   _stream_ptr(stream))
    if rc != TTT_OK:
        raise TttAttnError(rc, ttt_attn_last_error())


def ttt_attn_bwd(params, q, k, v, o, lse, d_o, cu_seqlens_dev, cu_seqlens_host, dq, dk, dv,
                 accumulate_dkv, workspace, stream=None):
    lib = load_library()
    K = params.k
    rc = lib.ttt_attn_bwd(ctypes.byref(params), _ptr_array(q, K), _ptr_array(k, K), _ptr_array(v, K),
                          _ptr_array(o, K), _ptr_array(lse, K), _ptr_array(d_o, K),
                          ctypes.c_void_p(cu_seqlens_dev.data_ptr()), _cu_host_array(cu_seqlens_host),
                          _ptr_array(dq, K), _ptr_array(dk, K), _ptr_array(dv, K), int(accumulate_dkv),
                          ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                          _stream_ptr(stream))
    if rc != TTT_OK:
        raise TttAttnError(rc, ttt_attn_last_error())


def ttt_loss_bwd_inplace(logits, target, grad, stream=None):
    """logits, target: [n_rows, vocab] device tensors of one dtype (fp32 or bf16), vocab contiguous;
    grad: [n_rows] fp32.  Overwrites `logits` with the gradient of the loss (Alg. 3)."""
    import torch
    lib = load_library()
    assert logits.dim() == 2 and target.shape == logits.shape and logits.dtype == target.dtype
    assert logits.stride(1) == 1 and target.stride(1) == 1 and grad.dtype == torch.float32 and grad.is_contiguous()
    dtype = {torch.float32: TTT_F32, torch.bfloat16: TTT_BF16}[logits.dtype]
    n, v = logits.shape
    rc = lib.ttt_loss_bwd_inplace(ctypes.c_void_p(logits.data_ptr()), ctypes.c_void_p(target.data_ptr()),
                                  ctypes.c_void_p(grad.data_ptr()), n, v, logits.stride(0) if n > 1 else max(logits.stride(0), v),
                                  target.stride(0) if n > 1 else max(target.stride(0), v), dtype, _stream_ptr(stream))
    if rc != TTT_OK:
        raise TttAttnError(rc, ttt_attn_last_error())


def ttt_qkv_rope_fwd(x, w, cos_tab, sin_tab, pos, q, k, v, stream=None):
    """x [T, Hin] and w [(hq + 2 hkv) d, Hin] bf16 (rows may be strided), cos_tab / sin_tab [n_pos, d/2] fp32,
    pos [T] int32; writes q [T, hq, d], k [T, hkv, d], v [T, hkv, d] (bf16, contiguous)."""
    import torch
    lib = load_library()
    T, hin = x.shape
    hq, d = q.shape[1], q.shape[2]
    hkv = k.shape[1]
    assert x.dtype == w.dtype == q.dtype == k.dtype == v.dtype == torch.bfloat16
    assert w.shape == ((hq + 2 * hkv) * d, hin) and x.stride(1) == 1 and w.stride(1) == 1
    assert q.is_contiguous() and k.is_contiguous() and v.is_contiguous() and k.shape == v.shape == (T, hkv, d)
    assert cos_tab.dtype == sin_tab.dtype == torch.float32 and cos_tab.is_contiguous() and sin_tab.is_contiguous()
    assert cos_tab.shape == sin_tab.shape and cos_tab.shape[1] == d // 2
    assert pos.dtype == torch.int32 and pos.is_contiguous() and pos.numel() == T
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    rc = lib.ttt_qkv_rope_fwd(p(x), p(w), p(cos_tab), p(sin_tab), p(pos), p(q), p(k), p(v), T, hin, hq, hkv, d,
                              x.stride(0) if T > 1 else max(x.stride(0), hin), w.stride(0), cos_tab.shape[0], TTT_BF16,
                              _stream_ptr(stream))
    if rc != TTT_OK:
        raise TttAttnError(rc, ttt_attn_last_error())


def ttt_o_proj_fwd(o, w, out, stream=None):
    """o [T, hq, d] (or [T, in]) and w [out_features, in] bf16, rows may be strided; writes out [T, out_features]."""
    import torch
    lib = load_library()
    o2 = o.reshape(o.shape[0], -1) if o.dim() == 3 else o
    T, fin = o2.shape
    assert o2.dtype == w.dtype == out.dtype == torch.bfloat16 and o2.stride(1) == 1 and w.stride(1) == 1
    assert w.shape[1] == fin and out.shape == (T, w.shape[0]) and out.is_contiguous()
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    rc = lib.ttt_o_proj_fwd(p(o2), p(w), p(out), T, fin, w.shape[0], o2.stride(0) if T > 1 else max(o2.stride(0), fin),
                            w.stride(0), TTT_BF16, _stream_ptr(stream))
    if rc != TTT_OK:
        raise TttAttnError(rc, ttt_attn_last_error())
