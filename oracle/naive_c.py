"""ctypes wrapper around oracle/spmm_naive.c.  TEST INFRASTRUCTURE ONLY.

build() compiles the C file with gcc (-O2, OpenMP, no fast-math);
spmm()/spmm_abs() run the naive masked triple loop on dense mask, dense W and
I, returning float64."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spmm_naive.c")
_LIB = os.path.join(_HERE, "liboracle_spmm.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.rbgp_oracle_threads.restype = ctypes.c_int
        lib.rbgp_oracle_spmm.restype = None
        lib.rbgp_oracle_spmm.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_long] * 3 + [ctypes.c_int]
        _lib = lib
    return _lib


def threads() -> int:
    return int(_load().rbgp_oracle_threads())


def _run(mask, W, I, take_abs):
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    W = np.ascontiguousarray(W, dtype=np.float32)
    I = np.ascontiguousarray(I, dtype=np.float32)
    M, K = mask.shape
    assert W.shape == (M, K) and I.shape[0] == K
    N = I.shape[1]
    O = np.empty((M, N), dtype=np.float64)
    _load().rbgp_oracle_spmm(mask.ctypes.data, W.ctypes.data, I.ctypes.data, O.ctypes.data,
                             M, K, N, int(take_abs))
    return O


def spmm(mask, W, I):
    return _run(mask, W, I, 0)


def spmm_abs(mask, W, I):
    return _run(mask, W, I, 1)
