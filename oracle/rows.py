"""ctypes front end of oracle/attn_rows.c (row-by-row fp64 attention oracle).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  `build()` compiles the C file with gcc into
oracle/liboracle_rows.so (beside its source); the functions below marshal numpy arrays and return fp64 results.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attn_rows.c")
_LIB = os.path.join(_HERE, "liboracle_rows.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.s1f_oracle_threads.restype = ctypes.c_int
    return _lib


def threads() -> int:
    return int(_load().s1f_oracle_threads())


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def _dims(q, k):
    hq, n, d = q.shape
    hkv = k.shape[0]
    assert k.shape == (hkv, n, d) and hq % hkv == 0
    return hq, hkv, n, d


def forward_rows(q, k, v, h: int, r0: int, r1: int):
    """(out [r1-r0, D], lse [r1-r0]) of rows r0..r1-1 of query head h of the full sequence."""
    q, qp = _f32(q); k, kp = _f32(k); v, vp = _f32(v)
    hq, hkv, n, d = _dims(q, k)
    assert 0 <= r0 <= r1 <= n and 0 <= h < hq
    out = np.empty((r1 - r0, d)); lse = np.empty(r1 - r0)
    _load().s1f_oracle_forward_rows(qp, kp, vp, hq, hkv, ctypes.c_int64(n), d, h, ctypes.c_int64(r0),
                                    ctypes.c_int64(r1), out.ctypes.data_as(ctypes.c_void_p),
                                    lse.ctypes.data_as(ctypes.c_void_p))
    return out, lse


def dq_rows(q, k, v, dout, h: int, r0: int, r1: int):
    """dq [r1-r0, D] of rows r0..r1-1 of query head h."""
    q, qp = _f32(q); k, kp = _f32(k); v, vp = _f32(v); dout, dp = _f32(dout)
    hq, hkv, n, d = _dims(q, k)
    assert 0 <= r0 <= r1 <= n and 0 <= h < hq
    dq = np.empty((r1 - r0, d))
    _load().s1f_oracle_dq_rows(qp, kp, vp, dp, hq, hkv, ctypes.c_int64(n), d, h, ctypes.c_int64(r0),
                               ctypes.c_int64(r1), dq.ctypes.data_as(ctypes.c_void_p))
    return dq


def dkdv_keys(q, k, v, dout, g: int, j0: int, j1: int):
    """(dk, dv) [j1-j0, D] of keys j0..j1-1 of K/V head g (summed over its query heads, all rows)."""
    q, qp = _f32(q); k, kp = _f32(k); v, vp = _f32(v); dout, dp = _f32(dout)
    hq, hkv, n, d = _dims(q, k)
    assert 0 <= j0 <= j1 <= n and 0 <= g < hkv
    dk = np.empty((j1 - j0, d)); dv = np.empty((j1 - j0, d))
    _load().s1f_oracle_dkdv_keys(qp, kp, vp, dp, hq, hkv, ctypes.c_int64(n), d, g, ctypes.c_int64(j0),
                                 ctypes.c_int64(j1), dk.ctypes.data_as(ctypes.c_void_p),
                                 dv.ctypes.data_as(ctypes.c_void_p))
    return dk, dv
