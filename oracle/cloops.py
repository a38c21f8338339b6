"""ctypes loader for oracle/loops.c -- TEST INFRASTRUCTURE ONLY.

``build()`` compiles the file with gcc (-O2, OpenMP, fp contraction off so that a*b+c
is two roundings as written); the functions below marshal numpy arrays to it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "loops.c")
_LIB = os.path.join(_HERE, "liboracle_loops.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC",
                               "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_max_threads.restype = ctypes.c_int
    return _lib


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def _ptr_array(arrays):
    arr = (ctypes.c_void_p * len(arrays))()
    for i, a in enumerate(arrays):
        assert a.flags["C_CONTIGUOUS"]
        arr[i] = a.ctypes.data
    return arr


def reduce_copy(srcs, dtype: str, ndst: int = 1, threads: int = 1):
    lib = _load()
    n = len(srcs[0])
    np_dt = np.float32 if dtype == "f32" else np.uint16
    srcs = [np.ascontiguousarray(s, dtype=np_dt) for s in srcs]
    dsts = [np.empty(n, dtype=np_dt) for _ in range(ndst)]
    fn = lib.oracle_reduce_copy_f32 if dtype == "f32" else lib.oracle_reduce_copy_bf16
    fn(_ptr_array(srcs), ctypes.c_int(len(srcs)), _ptr_array(dsts), ctypes.c_int(ndst),
       ctypes.c_int64(n), ctypes.c_int(threads))
    return dsts


def gather_copy(srcs, ndst: int = 1, threads: int = 1):
    lib = _load()
    srcs = [np.ascontiguousarray(s) for s in srcs]
    nbytes = srcs[0].nbytes
    dsts = [np.empty(len(srcs[0]) * len(srcs), dtype=srcs[0].dtype) for _ in range(ndst)]
    lib.oracle_gather_copy(_ptr_array(srcs), ctypes.c_int(len(srcs)), _ptr_array(dsts), ctypes.c_int(ndst),
                           ctypes.c_int64(nbytes), ctypes.c_int(threads))
    return dsts


def gemm(a_bits, b_bits, b_is_nk: bool = True, row_lo: int = 0, row_hi=None, threads: int = 1):
    """fp64 C rows [row_lo, row_hi); returns an array of shape (row_hi - row_lo, N)."""
    lib = _load()
    a = np.ascontiguousarray(a_bits, dtype=np.uint16)
    b = np.ascontiguousarray(b_bits, dtype=np.uint16)
    M, K = a.shape
    N = b.shape[0] if b_is_nk else b.shape[1]
    row_hi = M if row_hi is None else row_hi
    out = np.zeros((row_hi - row_lo, N), dtype=np.float64)
    lib.oracle_gemm_bf16(ctypes.c_void_p(a.ctypes.data), ctypes.c_void_p(b.ctypes.data),
                         ctypes.c_void_p(out.ctypes.data), ctypes.c_int64(M), ctypes.c_int64(N), ctypes.c_int64(K),
                         ctypes.c_int(1 if b_is_nk else 0), ctypes.c_int64(row_lo), ctypes.c_int64(row_hi),
                         ctypes.c_int(threads))
    return out
