"""ctypes loader for ``brute_force.c`` (scalar-loop attention for tiny shapes).

TEST INFRASTRUCTURE ONLY.  ``build()`` compiles the C file with gcc next to this module.
"""
from __future__ import annotations

import ctypes
import pathlib
import subprocess

import numpy as np

_HERE = pathlib.Path(__file__).resolve().parent
_SO = _HERE / "libbrute_force.so"
_lib = None


def build(force: bool = True) -> pathlib.Path:
    src = _HERE / "brute_force.c"
    if force or not _SO.exists() or _SO.stat().st_mtime < src.stat().st_mtime:
        subprocess.run(["gcc", "-O2", "-fPIC", "-shared", "-o", str(_SO), str(src), "-lm"], check=True)
    return _SO


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = ctypes.CDLL(str(_SO))
        dp = ctypes.POINTER(ctypes.c_double)
        _lib.brute_attn_fwd.argtypes = [dp] * 5 + [ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_int]
        _lib.brute_attn_bwd.argtypes = [dp] * 7 + [ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_int]
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def head_forward(q, k, v, scale, causal=True):
    q, k, v = (np.ascontiguousarray(x, dtype=np.float64) for x in (q, k, v))
    S, D = q.shape
    o = np.empty((S, D)); lse = np.empty(S)
    rc = _load().brute_attn_fwd(_p(q), _p(k), _p(v), _p(o), _p(lse), S, D, float(scale), int(causal))
    assert rc == 0
    return o, lse


def head_backward(q, k, v, g, scale, causal=True):
    q, k, v, g = (np.ascontiguousarray(x, dtype=np.float64) for x in (q, k, v, g))
    S, D = q.shape
    dq = np.empty((S, D)); dk = np.empty((S, D)); dv = np.empty((S, D))
    rc = _load().brute_attn_bwd(_p(q), _p(k), _p(v), _p(g), _p(dq), _p(dk), _p(dv), S, D, float(scale), int(causal))
    assert rc == 0
    return dq, dk, dv
