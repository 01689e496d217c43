"""ctypes front end of the C oracle (attn_oracle.c) -- TEST INFRASTRUCTURE ONLY.

Exact softmax attention (paper Eq. 1, Sec. 3.1; causal mask, Sec. 4.3; optional full-attention
spans of multimodal inputs, Sec. 4.3 time estimation) and its gradients, fp64, per unsharded
sequence.  Inputs are bf16 bit patterns.  `span_id` [T] int32 marks tokens (>= 0) that see every
token of the same sequence with the same id; None or -1 everywhere is the causal mask.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attn_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile attn_oracle.c with gcc (plain C + OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        P, I, L, D = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_double
        lib.oracle_attn_fwd.argtypes = [P, P, P, P, I, I, I, I, D, P, P, L, P, P]
        lib.oracle_attn_fwd.restype = None
        lib.oracle_attn_dq.argtypes = [P, P, P, P, P, I, I, I, I, D, P, P, L, P, P, P]
        lib.oracle_attn_dq.restype = None
        lib.oracle_attn_dkv.argtypes = [P, P, P, P, P, I, L, I, I, I, D, P, P, L, P, P, P, L, P, P]
        lib.oracle_attn_dkv.restype = None
        lib.oracle_num_threads.restype = I
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _chk(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _span(span_id, T):
    """(keep-alive array, pointer) of the optional span ids"""
    if span_id is None:
        return None, None
    a = _chk(span_id, np.int32)
    assert a.shape == (T,)
    return a, _p(a)


def attn_fwd(q, k, v, cu_seqlens, scale, rows=None, span_id=None):
    """q [T,Hq,D], k,v [T,Hkv,D] uint16 bf16 bits.  Returns O [n_rows,Hq,D], LSE [n_rows,Hq] (fp64)."""
    q, k, v = _chk(q, np.uint16), _chk(k, np.uint16), _chk(v, np.uint16)
    cu = _chk(cu_seqlens, np.int32)
    T, hq, D = q.shape
    hkv = k.shape[1]
    assert k.shape == (T, hkv, D) and v.shape == (T, hkv, D) and hq % hkv == 0
    assert cu[0] == 0 and cu[-1] == T
    rows = np.arange(T, dtype=np.int64) if rows is None else _chk(rows, np.int64)
    O = np.empty((len(rows), hq, D), np.float64)
    LSE = np.empty((len(rows), hq), np.float64)
    sp, sp_p = _span(span_id, T)
    _load().oracle_attn_fwd(_p(q), _p(k), _p(v), _p(cu), len(cu) - 1, hq, hkv, D, float(scale), sp_p,
                            _p(rows), len(rows), _p(O), _p(LSE))
    return O, LSE


def attn_dq(q, k, v, d_o, cu_seqlens, scale, rows, O, LSE, span_id=None):
    """dQ [n_rows,Hq,D] for the listed rows; O, LSE are the oracle's forward results for them."""
    q, k, v, d_o = (_chk(x, np.uint16) for x in (q, k, v, d_o))
    cu = _chk(cu_seqlens, np.int32)
    T, hq, D = q.shape
    hkv = k.shape[1]
    rows = _chk(rows, np.int64)
    O, LSE = _chk(O, np.float64), _chk(LSE, np.float64)
    assert O.shape == (len(rows), hq, D) and LSE.shape == (len(rows), hq)
    dQ = np.empty((len(rows), hq, D), np.float64)
    sp, sp_p = _span(span_id, T)
    _load().oracle_attn_dq(_p(q), _p(k), _p(v), _p(d_o), _p(cu), len(cu) - 1, hq, hkv, D, float(scale), sp_p,
                           _p(rows), len(rows), _p(O), _p(LSE), _p(dQ))
    return dQ


def attn_dkv(q, k, v, d_o, cu_seqlens, scale, rows, O, LSE, keys=None, span_id=None):
    """dK, dV summed over the listed query rows, for the listed keys (all T tokens if None)."""
    q, k, v, d_o = (_chk(x, np.uint16) for x in (q, k, v, d_o))
    cu = _chk(cu_seqlens, np.int32)
    T, hq, D = q.shape
    hkv = k.shape[1]
    rows = _chk(rows, np.int64)
    O, LSE = _chk(O, np.float64), _chk(LSE, np.float64)
    assert O.shape == (len(rows), hq, D) and LSE.shape == (len(rows), hq)
    nk = T if keys is None else len(keys)
    keys_a = None if keys is None else _chk(keys, np.int64)
    dK = np.empty((nk, hkv, D), np.float64)
    dV = np.empty((nk, hkv, D), np.float64)
    sp, sp_p = _span(span_id, T)
    _load().oracle_attn_dkv(_p(q), _p(k), _p(v), _p(d_o), _p(cu), len(cu) - 1, T, hq, hkv, D, float(scale), sp_p,
                            _p(rows), len(rows), _p(O), _p(LSE), None if keys_a is None else _p(keys_a), nk,
                            _p(dK), _p(dV))
    return dK, dV


def attn_bwd(q, k, v, d_o, cu_seqlens, scale, rows=None, O=None, LSE=None, want_dkv=True, span_id=None):
    """Gradients of sum(O*dO).  Returns dQ [n_rows,Hq,D], dK, dV [T,Hkv,D] (fp64); dK/dV are
    summed over the listed query rows only."""
    T = np.asarray(q).shape[0]
    rows = np.arange(T, dtype=np.int64) if rows is None else _chk(rows, np.int64)
    if O is None or LSE is None:
        O, LSE = attn_fwd(q, k, v, cu_seqlens, scale, rows, span_id)
    dQ = attn_dq(q, k, v, d_o, cu_seqlens, scale, rows, O, LSE, span_id)
    if not want_dkv:
        return dQ, None, None
    dK, dV = attn_dkv(q, k, v, d_o, cu_seqlens, scale, rows, O, LSE, span_id=span_id)
    return dQ, dK, dV
