"""ctypes front end of the fp64 CPU oracle (``svdmlp_oracle.c``).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this module;
only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` do.  It shares no code with the HIP path.

The oracle evaluates, in IEEE double and with no intermediate rounding,

    linear:  O = (X U) V                                   (paper Sec. 3.1, Eq. 1)
    gated :  Z = ((SiLU((X Ug) Vg) .* ((X Uu) Vu)) Ud) Vd  (paper Sec. 4.2.2, Alg. 2, Alg. 3)

Inputs are numpy float64 arrays (values already rounded to the storage type of
the GPU path are passed in exactly).  Every function here is pinned by
``tests/test_oracle_pins.py``; none is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "svdmlp_oracle.c"
_LIB = _HERE / "libsvdmlp_oracle.so"
_lib = None


def build(force: bool = False) -> Path:
    """Compile the C oracle with gcc (OpenMP, -O2; no fast-math, so IEEE semantics hold)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        cmd = ["gcc", "-O2", "-ftree-vectorize", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               "-ffp-contract=off", "-o", str(_LIB), str(_SRC), "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_LIB))
        dp = ctypes.POINTER(ctypes.c_double)
        i64 = ctypes.c_int64
        lib.svdmlp_oracle_linear.argtypes = [dp, i64, i64, i64, i64, dp, dp, dp]
        lib.svdmlp_oracle_linear.restype = ctypes.c_int
        lib.svdmlp_oracle_gated.argtypes = [dp, i64, i64, i64, i64, i64, dp, dp, dp, dp, dp, dp, dp, dp]
        lib.svdmlp_oracle_gated.restype = ctypes.c_int
        lib.svdmlp_oracle_silu.argtypes = [ctypes.c_double]
        lib.svdmlp_oracle_silu.restype = ctypes.c_double
        lib.svdmlp_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f64(a, shape=None) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float64)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def threads() -> int:
    """Number of host threads the oracle's row loop will use."""
    return int(_load().svdmlp_oracle_threads())


def silu(x: float) -> float:
    """SiLU(x) = x / (1 + exp(-x)) in double (epilogue of Alg. 3)."""
    return float(_load().svdmlp_oracle_silu(float(x)))


def linear(X, U, V) -> np.ndarray:
    """O = (X U) V with X[M,K], U[K,r], V[r,N] (paper Sec. 3.1; block form Eq. 1)."""
    X = _f64(X)
    M, K = X.shape
    U = _f64(U)
    r = U.shape[1]
    U = _f64(U, (K, r))
    V = _f64(V)
    N = V.shape[1]
    V = _f64(V, (r, N))
    O = np.empty((M, N), dtype=np.float64)
    rc = _load().svdmlp_oracle_linear(_ptr(X), M, K, N, r, _ptr(U), _ptr(V), _ptr(O))
    if rc != 0:
        raise RuntimeError(f"svdmlp_oracle_linear failed ({rc})")
    return O


def gated(X, Ug, Vg, Uu, Vu, Ud, Vd, return_H: bool = False):
    """Z = ((SiLU((X Ug) Vg) .* ((X Uu) Vu)) Ud) Vd (paper Alg. 2 with Alg. 3's epilogue).

    Shapes: X[M,K], Ug/Uu[K,r], Vg/Vu[r,N], Ud[N,r2], Vd[r2,K]; returns Z[M,K]
    (and H[M,N] when ``return_H``).
    """
    X = _f64(X)
    M, K = X.shape
    Ug = _f64(Ug)
    r = Ug.shape[1]
    Ug = _f64(Ug, (K, r))
    Uu = _f64(Uu, (K, r))
    Vg = _f64(Vg)
    N = Vg.shape[1]
    Vg = _f64(Vg, (r, N))
    Vu = _f64(Vu, (r, N))
    Ud = _f64(Ud)
    r2 = Ud.shape[1]
    Ud = _f64(Ud, (N, r2))
    Vd = _f64(Vd, (r2, K))
    Z = np.empty((M, K), dtype=np.float64)
    H = np.empty((M, N), dtype=np.float64) if return_H else None
    rc = _load().svdmlp_oracle_gated(_ptr(X), M, K, N, r, r2, _ptr(Ug), _ptr(Vg), _ptr(Uu), _ptr(Vu),
                                     _ptr(Ud), _ptr(Vd), _ptr(Z), _ptr(H) if return_H else None)
    if rc != 0:
        raise RuntimeError(f"svdmlp_oracle_gated failed ({rc})")
    return (Z, H) if return_H else Z
