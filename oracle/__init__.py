"""CPU oracle for the causal long convolution (float64, direct O(N^2) sums).

TEST INFRASTRUCTURE ONLY: nothing on the product path may import this package.
Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline``
leg use it.  It shares no code with the HIP library and does not import it.

The arithmetic lives in ``oracle.c`` (paper Eq. 1 / Algorithm 1 line 4 and the
exact adjoints of that bilinear map); this module compiles that file with gcc,
loads it with ctypes and marshals numpy arrays.  Every pin of the oracle
(closed forms, brute-force DFT route of Eq. 2 on tiny N, adjoint identities,
finite differences) is in ``tests/test_oracle.py``; no output is unpinned.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile oracle.c into liboracle.so (gcc, OpenMP). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        i64 = ctypes.c_int64
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_longconv_fwd.argtypes = [dp, dp, dp, dp, i64, i64, i64]
        lib.oracle_longconv_bwd_du.argtypes = [dp, dp, dp, dp, i64, i64, i64]
        lib.oracle_longconv_bwd_dk_dD.argtypes = [dp, dp, dp, dp, i64, i64, i64]
        lib.oracle_longconv_bwd.argtypes = [dp, dp, dp, dp, dp, dp, dp, i64, i64, i64]
        for f in (lib.oracle_longconv_fwd, lib.oracle_longconv_bwd_du,
                  lib.oracle_longconv_bwd_dk_dD, lib.oracle_longconv_bwd):
            f.restype = None
        _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the C oracle will use (OpenMP max threads)."""
    return int(_load().oracle_num_threads())


def _f64(a, shape):
    a = np.ascontiguousarray(np.asarray(a, dtype=np.float64))
    if a.shape != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {a.shape}")
    return a


def _p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def longconv_fwd(u, k, D):
    """y[b,h,t] = sum_{s<=t} k[h,s] u[b,h,t-s] + D[h] u[b,h,t]  (Eq. 1, Alg. 1 line 4)."""
    u = np.asarray(u)
    B, H, N = u.shape
    u = _f64(u, (B, H, N)); k = _f64(k, (H, N)); D = _f64(D, (H,))
    y = np.empty_like(u)
    _load().oracle_longconv_fwd(_p(u), _p(k), _p(D), _p(y), B, H, N)
    return y


def longconv_bwd(dy, u, k, D):
    """Exact adjoints of longconv_fwd: returns (du [B,H,N], dk [H,N], dD [H])."""
    u = np.asarray(u)
    B, H, N = u.shape
    dy = _f64(dy, (B, H, N)); u = _f64(u, (B, H, N)); k = _f64(k, (H, N)); D = _f64(D, (H,))
    du = np.empty_like(u); dk = np.empty((H, N)); dD = np.empty((H,))
    _load().oracle_longconv_bwd(_p(dy), _p(u), _p(k), _p(D), _p(du), _p(dk), _p(dD), B, H, N)
    return du, dk, dD


def longconv_bwd_du(dy, k, D):
    """du only (rows are independent, so any subset of rows may be passed)."""
    dy = np.asarray(dy)
    B, H, N = dy.shape
    dy = _f64(dy, (B, H, N)); k = _f64(k, (H, N)); D = _f64(D, (H,))
    du = np.empty_like(dy)
    _load().oracle_longconv_bwd_du(_p(dy), _p(k), _p(D), _p(du), B, H, N)
    return du


def longconv_bwd_dk_dD(dy, u):
    """dk, dD only (heads are independent; pass all batch rows of the chosen heads)."""
    u = np.asarray(u)
    B, H, N = u.shape
    dy = _f64(dy, (B, H, N)); u = _f64(u, (B, H, N))
    dk = np.empty((H, N)); dD = np.empty((H,))
    _load().oracle_longconv_bwd_dk_dD(_p(dy), _p(u), _p(dk), _p(dD), B, H, N)
    return dk, dD
