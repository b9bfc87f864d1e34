"""CPU oracle package.  TEST INFRASTRUCTURE ONLY.

Only `tests/`, `__graft_entry__.smoke()` and the `cpu_baseline` leg of
`bench.py` may import this package.  The GPU library never does, and this
package never imports the GPU library.

  la_oracle.py   NumPy fp64: quadratic masked form and token recurrence
  la_oracle.c    compiled fp64 token recurrence (OpenMP over independent scans)
  build_oracle   compiles la_oracle.c into libla_oracle.so beside the source
  c_recurrence_* ctypes wrappers over the compiled recurrence
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

from .la_oracle import (decay_matrix, decode_step, gate_norm_bwd, gate_norm_fwd, left_product_bwd,
                        left_product_fwd, lrpe_features, lrpe_features_bwd, lrpe_fwd, recurrence_bwd, recurrence_fwd, rel_max_err, swish,
                        swish_attention_bwd, swish_attention_fwd, swish_grad)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "la_oracle.c")
_LIB = os.path.join(_HERE, "libla_oracle.so")
_lib = None


def build_oracle(force: bool = False) -> str:
    """Compile la_oracle.c with gcc (fp64, -O3, OpenMP).  No fast-math: the
    order of operations stays as written."""
    if force or (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build_oracle()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.la_oracle_recurrence_fwd.argtypes = [dp, dp, dp, dp, dp,
                                                 ctypes.c_long, ctypes.c_long, ctypes.c_long]
        lib.la_oracle_recurrence_fwd.restype = ctypes.c_int
        lib.la_oracle_recurrence_bwd.argtypes = [dp] * 8 + [ctypes.c_long] * 3
        lib.la_oracle_recurrence_bwd.restype = ctypes.c_int
        lib.la_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def oracle_threads() -> int:
    return int(_load().la_oracle_threads())


def _p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _flat(x):
    x = np.ascontiguousarray(np.asarray(x, dtype=np.float64))
    B, H, n, d = x.shape
    return x.reshape(B * H, n, d)


def c_recurrence_fwd(Q, K, V, lam):
    """Compiled recurrence, forward.  Q, K, V: [B, H, n, d]; lam: [H]."""
    B, H, n, d = np.asarray(Q).shape
    q, k, v = _flat(Q), _flat(K), _flat(V)
    l = np.ascontiguousarray(np.tile(np.asarray(lam, dtype=np.float64), B))
    o = np.empty_like(q)
    rc = _load().la_oracle_recurrence_fwd(_p(q), _p(k), _p(v), _p(l), _p(o), B * H, n, d)
    if rc != 0:
        raise MemoryError("la_oracle_recurrence_fwd")
    return o.reshape(B, H, n, d)


def c_recurrence_bwd(Q, K, V, lam, dO):
    """Compiled recurrence, backward.  Returns (dQ, dK, dV)."""
    B, H, n, d = np.asarray(Q).shape
    q, k, v, g = _flat(Q), _flat(K), _flat(V), _flat(dO)
    l = np.ascontiguousarray(np.tile(np.asarray(lam, dtype=np.float64), B))
    dq, dk, dv = np.empty_like(q), np.empty_like(q), np.empty_like(q)
    rc = _load().la_oracle_recurrence_bwd(_p(q), _p(k), _p(v), _p(l), _p(g),
                                          _p(dq), _p(dk), _p(dv), B * H, n, d)
    if rc != 0:
        raise MemoryError("la_oracle_recurrence_bwd")
    shp = (B, H, n, d)
    return dq.reshape(shp), dk.reshape(shp), dv.reshape(shp)
