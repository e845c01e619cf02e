"""ctypes access to fp64_soft_add.c and fp64_soft_mul.c (oracle; test infrastructure).

`build()` compiles the C files with gcc into oracle/_build/; `soft_add(x, y)` / `soft_mul(x, y)` combine two
float64 arrays element by element with the integer-only addition / multiplication and return float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, "fp64_soft_add.c"), os.path.join(_HERE, "fp64_soft_mul.c")]
_LIB = os.path.join(_HERE, "_build", "liboracle_softfloat.so")
_lib = None


def build(force: bool = False) -> str:
    os.makedirs(os.path.dirname(_LIB), exist_ok=True)
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(p) for p in _SRCS):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-shared", "-fPIC", "-o", _LIB] + _SRCS)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_fp64_add_array.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t]
        _lib.oracle_fp64_add_array.restype = None
        _lib.oracle_fp64_add_bits.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
        _lib.oracle_fp64_add_bits.restype = ctypes.c_uint64
        _lib.oracle_fp64_mul_array.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t]
        _lib.oracle_fp64_mul_array.restype = None
        _lib.oracle_fp64_mul_bits.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
        _lib.oracle_fp64_mul_bits.restype = ctypes.c_uint64
    return _lib


def soft_add(x: np.ndarray, y: np.ndarray) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    x, y = np.broadcast_arrays(x, y)
    xa = np.ascontiguousarray(x)
    ya = np.ascontiguousarray(y)
    out = np.empty(xa.shape, dtype=np.float64)
    _load().oracle_fp64_add_array(xa.ctypes.data, ya.ctypes.data, out.ctypes.data, xa.size)
    return out


def soft_add_bits(a: int, b: int) -> int:
    return int(_load().oracle_fp64_add_bits(a, b))


def soft_mul(x: np.ndarray, y: np.ndarray) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    x, y = np.broadcast_arrays(x, y)
    xa = np.ascontiguousarray(x)
    ya = np.ascontiguousarray(y)
    out = np.empty(xa.shape, dtype=np.float64)
    _load().oracle_fp64_mul_array(xa.ctypes.data, ya.ctypes.data, out.ctypes.data, xa.size)
    return out


def soft_mul_bits(a: int, b: int) -> int:
    return int(_load().oracle_fp64_mul_bits(a, b))
