"""TEST INFRASTRUCTURE ONLY: ctypes front end of the plain-C fp64 oracle (ttt_oracle.c).

Argument marshalling only; every number is produced by the C file.  Inputs are numpy arrays of
float32 (exact images of bf16/fp32 tensors) or float64 (finite-difference tests); all arithmetic is
fp64.  Layouts: Q [k,T,hq,d]; K,V [k,T,hkv,d]; cotangent dO_rows [n_rows,hq,d] for the listed rows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ttt_oracle.c")
_INC = os.path.join(_HERE, "ttt_oracle_core.inc")
_BUILD = os.path.join(_HERE, "_build")
_LIB = os.path.join(_BUILD, "libttt_oracle.so")
_lock = threading.Lock()
_lib = None


class _Shape(ctypes.Structure):
    _fields_ = [("k", ctypes.c_int32), ("T", ctypes.c_int32), ("n_docs", ctypes.c_int32),
                ("hq", ctypes.c_int32), ("hkv", ctypes.c_int32), ("d", ctypes.c_int32),
                ("scale", ctypes.c_double)]


def build_oracle(force: bool = False) -> str:
    """Compile ttt_oracle.c with gcc (OpenMP) into oracle/_build/ and return the library path."""
    os.makedirs(_BUILD, exist_ok=True)
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_INC)))
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        cmd = ["gcc", "-O3", "-march=native", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True, cwd=_HERE)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build_oracle())
            for name in ("ttt_oracle_run_f32in", "ttt_oracle_run_f64in"):
                fn = getattr(lib, name)
                fn.restype = ctypes.c_int
                fn.argtypes = [ctypes.POINTER(_Shape), ctypes.c_void_p,
                               ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                               ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                               ctypes.c_void_p,
                               ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                               ctypes.c_void_p, ctypes.c_void_p]
            lib.ttt_oracle_mask_row.restype = None
            lib.ttt_oracle_mask_row.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                ctypes.c_void_p, ctypes.c_void_p]
            _lib = lib
    return _lib


@dataclass
class OracleResult:
    rows: np.ndarray            # [n_rows, 2] (step, token)
    O: np.ndarray               # [n_rows, hq, d] float64
    LSE: np.ndarray             # [n_rows, hq]
    dQ: np.ndarray | None       # [n_rows, hq, d]
    dK: np.ndarray | None       # [k, T, hkv, d], summed over the listed rows
    dV: np.ndarray | None


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def oracle_run(Q, K, V, cu_seqlens, scale, row_step, row_tok, dO_rows=None) -> OracleResult:
    """Forward (and, if dO_rows is given, backward) for the listed query rows."""
    lib = _load()
    dt = Q.dtype
    assert dt in (np.float32, np.float64)
    Q = np.ascontiguousarray(Q, dtype=dt); K = np.ascontiguousarray(K, dtype=dt)
    V = np.ascontiguousarray(V, dtype=dt)
    k, T, hq, d = Q.shape
    hkv = K.shape[2]
    assert K.shape == (k, T, hkv, d) and V.shape == (k, T, hkv, d)
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    row_step = np.ascontiguousarray(row_step, dtype=np.int32)
    row_tok = np.ascontiguousarray(row_tok, dtype=np.int32)
    n = int(row_step.shape[0])
    assert row_tok.shape == (n,)
    sh = _Shape(k, T, len(cu) - 1, hq, hkv, d, float(scale))
    O = np.empty((n, hq, d), dtype=np.float64)
    LSE = np.empty((n, hq), dtype=np.float64)
    dQ = dK = dV = None
    if dO_rows is not None:
        dO_rows = np.ascontiguousarray(dO_rows, dtype=dt)
        assert dO_rows.shape == (n, hq, d)
        dQ = np.empty((n, hq, d), dtype=np.float64)
        dK = np.empty((k, T, hkv, d), dtype=np.float64)
        dV = np.empty((k, T, hkv, d), dtype=np.float64)
    fn = lib.ttt_oracle_run_f32in if dt == np.float32 else lib.ttt_oracle_run_f64in
    rc = fn(ctypes.byref(sh), _ptr(cu), _ptr(Q), _ptr(K), _ptr(V), n, _ptr(row_step), _ptr(row_tok),
            _ptr(dO_rows), _ptr(O), _ptr(LSE), _ptr(dQ), _ptr(dK), _ptr(dV))
    if rc != 0:
        raise ValueError(f"ttt_oracle_run rejected its arguments (code {rc})")
    return OracleResult(np.stack([row_step, row_tok], axis=1), O, LSE, dQ, dK, dV)


def oracle_full(Q, K, V, cu_seqlens, scale, dO=None, step_begin=0, step_end=None):
    """All rows of steps [step_begin, step_end).  dO is [k,T,hq,d] (only the steps in range are read).

    Returns O [n_steps,T,hq,d], LSE [n_steps,hq,T], dQ [n_steps,T,hq,d], dK, dV [k,T,hkv,d]
    (the last two hold the sums over the steps in range)."""
    k, T, hq, d = Q.shape
    step_end = k if step_end is None else step_end
    ns = step_end - step_begin
    row_step = np.repeat(np.arange(step_begin, step_end, dtype=np.int32), T)
    row_tok = np.tile(np.arange(T, dtype=np.int32), ns)
    dO_rows = None if dO is None else np.ascontiguousarray(dO[step_begin:step_end]).reshape(ns * T, hq, d)
    r = oracle_run(Q, K, V, cu_seqlens, scale, row_step, row_tok, dO_rows)
    O = r.O.reshape(ns, T, hq, d)
    LSE = np.ascontiguousarray(r.LSE.reshape(ns, T, hq).transpose(0, 2, 1))
    dQ = None if r.dQ is None else r.dQ.reshape(ns, T, hq, d)
    return O, LSE, dQ, r.dK, r.dV


def oracle_mask(k, cu_seqlens):
    """Explicit boolean mask [k*T, k*T] (query slot j*T+i, key slot l*T+m) from the C predicate."""
    lib = _load()
    cu = np.asarray(cu_seqlens, dtype=np.int32)
    T = int(cu[-1])
    tok_doc = np.ascontiguousarray(np.repeat(np.arange(len(cu) - 1, dtype=np.int32), np.diff(cu)))
    M = np.zeros((k * T, k * T), dtype=np.uint8)
    for j in range(k):
        for i in range(T):
            row = M[j * T + i]
            lib.ttt_oracle_mask_row(j, i, k, T, _ptr(tok_doc), _ptr(row))
    return M.astype(bool)
