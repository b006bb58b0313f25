"""Build and call the plain-C hard-ECC oracle.  TEST INFRASTRUCTURE ONLY.

``build()`` compiles ``ecc_oracle_c.c`` with gcc (-O2 -fopenmp) into
``oracle/libecc_oracle.so``; the wrappers below marshal numpy arrays.  Nothing
here touches the HIP library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ecc_oracle_c.c")
_SO = os.path.join(_HERE, "libecc_oracle.so")
_lib = None

_DT = {np.dtype(np.uint8): 0, np.dtype(np.uint16): 1, np.dtype(np.float32): 2}


def build(force: bool = False) -> str:
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _SO, _SRC])
    return _SO


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_SO)
        i64 = ctypes.c_int64
        _lib.ecc_oracle_coeff.argtypes = [ctypes.c_void_p, ctypes.c_int, i64, i64, i64,
                                          ctypes.c_void_p]
        _lib.ecc_oracle_hard.argtypes = [ctypes.c_void_p, ctypes.c_int, i64, i64, i64, i64,
                                         ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        _lib.ecc_oracle_threads.restype = ctypes.c_int
    return _lib


def _dhw(shape):
    if len(shape) == 2:
        return 1, shape[0], shape[1]
    if len(shape) == 3:
        return shape
    raise ValueError("grid must be 2D or 3D")


def threads() -> int:
    return int(_load().ecc_oracle_threads())


def coeff(X: np.ndarray) -> np.ndarray:
    X = np.ascontiguousarray(X)
    D, H, W = _dhw(X.shape)
    out = np.empty(X.shape, dtype=np.int8)
    _load().ecc_oracle_coeff(X.ctypes.data, _DT[X.dtype], D, H, W, out.ctypes.data)
    return out


def ecc_hard_batch(Xb: np.ndarray, t: np.ndarray) -> np.ndarray:
    """Xb: [batch, (D,) H, W]; t: float64 thresholds; returns int64 [batch, bins]."""
    Xb = np.ascontiguousarray(Xb)
    t = np.ascontiguousarray(t, dtype=np.float64)
    D, H, W = _dhw(Xb.shape[1:])
    out = np.empty((Xb.shape[0], len(t)), dtype=np.int64)
    _load().ecc_oracle_hard(Xb.ctypes.data, _DT[Xb.dtype], D, H, W, Xb.shape[0], len(t),
                            t.ctypes.data, out.ctypes.data)
    return out


def ecc_hard(X: np.ndarray, t: np.ndarray) -> np.ndarray:
    return ecc_hard_batch(np.ascontiguousarray(X)[None], t)[0]
