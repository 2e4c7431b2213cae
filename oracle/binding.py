"""ctypes access to the C oracle (oracle/svd_oracle.c).

Test infrastructure only: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg, never by the HIP library or its binding.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "svd_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

_i64 = ctypes.c_int64
_dp = ctypes.POINTER(ctypes.c_double)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2 -fopenmp, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               "-fno-fast-math", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.orc_num_threads.restype = ctypes.c_int
        lib.orc_householder.argtypes = [_i64, _dp, _dp, _i64, _dp]
        lib.orc_householder.restype = None
        lib.orc_bidiagonalize.argtypes = [_i64, _i64, _dp, _i64, _dp, _dp, _dp, _dp]
        lib.orc_bidiagonalize.restype = ctypes.c_int
        lib.orc_bdsvals.argtypes = [_i64, _dp, _dp, _dp]
        lib.orc_bdsvals.restype = ctypes.c_int
        lib.orc_svdvals.argtypes = [_i64, _i64, _dp, _i64, _dp]
        lib.orc_svdvals.restype = ctypes.c_int
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(_dp)


def num_threads() -> int:
    return int(_load().orc_num_threads())


def householder(x: np.ndarray):
    """Reflector for the vector x: returns (beta, v, tau) with v[0] = 1."""
    x = np.array(x, dtype=np.float64)
    n = x.size
    alpha = ctypes.c_double(x[0] if n else 0.0)
    tail = np.ascontiguousarray(x[1:]) if n > 1 else np.zeros(1)
    tau = ctypes.c_double(0.0)
    _load().orc_householder(n, ctypes.byref(alpha), _ptr(tail), 1, ctypes.byref(tau))
    v = np.concatenate([[1.0], tail[:max(n - 1, 0)]]) if n else np.zeros(0)
    return alpha.value, v, tau.value


def bidiagonalize(a: np.ndarray):
    """Returns (d, e, factored, tauq, taup) for the m x n (m >= n) matrix a."""
    f = np.array(a, dtype=np.float64, order="F")
    m, n = f.shape
    d = np.zeros(max(n, 1))
    e = np.zeros(max(n, 1))
    tq = np.zeros(max(n, 1))
    tp = np.zeros(max(n, 1))
    rc = _load().orc_bidiagonalize(m, n, _ptr(f), max(m, 1), _ptr(d), _ptr(e), _ptr(tq), _ptr(tp))
    if rc != 0:
        raise ValueError(f"orc_bidiagonalize failed with {rc}")
    return d[:n], e[:max(n - 1, 0)], f, tq[:n], tp[:max(n - 1, 0)]


def bdsvals(d, e) -> np.ndarray:
    d = np.ascontiguousarray(d, dtype=np.float64)
    e = np.ascontiguousarray(e, dtype=np.float64)
    n = d.size
    if e.size != max(n - 1, 0):
        raise ValueError("e must have n-1 entries")
    ebuf = e if e.size else np.zeros(1)
    s = np.zeros(max(n, 1))
    rc = _load().orc_bdsvals(n, _ptr(d if n else np.zeros(1)), _ptr(ebuf), _ptr(s))
    if rc != 0:
        raise ValueError(f"orc_bdsvals failed with {rc}")
    return s[:n]


def svdvals(a: np.ndarray) -> np.ndarray:
    """Singular values (descending, fp64) of a; the input is converted to fp64
    and left untouched."""
    f = np.array(a, dtype=np.float64, order="F")
    m, n = f.shape
    if m < n:
        f = np.asfortranarray(f.T)
        m, n = n, m
    s = np.zeros(max(n, 1))
    rc = _load().orc_svdvals(m, n, _ptr(f), max(m, 1), _ptr(s))
    if rc != 0:
        raise ValueError(f"orc_svdvals failed with {rc}")
    return s[:n]
