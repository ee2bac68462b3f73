"""ctypes front end of ``matmul.c`` -- TEST INFRASTRUCTURE ONLY.

``matmul(A, B)`` is ``C = A B`` by definition (Section 2.1) in fp64;
``reduce_replicas(parts)`` is the fp32 left-to-right replica sum (Table 1).
``build()`` compiles the C file with gcc; loading builds it when the shared
object is missing.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "matmul.c")
_LIB = os.path.join(_HERE, "liboracle_matmul.so")
_lib = None

F64, F32, BF16 = 0, 1, 2


def build() -> str:
    """Compile matmul.c.  No -ffast-math and no contraction: the sums keep the
    order and rounding that the source states.  x86-64-v3 rather than native so
    that the object runs on whatever host the GPU machine has."""
    cmd = ["gcc", "-O3", "-march=x86-64-v3", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
           "-std=c11", "-Wall", "-o", _LIB, _SRC]
    subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
            build()
        lib = ctypes.CDLL(_LIB)
        lib.oracle_matmul.restype = ctypes.c_int
        lib.oracle_matmul.argtypes = [ctypes.c_int,
                                      ctypes.c_void_p, ctypes.c_int64,
                                      ctypes.c_void_p, ctypes.c_int64,
                                      ctypes.c_void_p, ctypes.c_int64,
                                      ctypes.c_int64, ctypes.c_int64, ctypes.c_int64]
        lib.oracle_reduce_replicas.restype = ctypes.c_int
        lib.oracle_reduce_replicas.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                                               ctypes.c_void_p, ctypes.c_int64,
                                               ctypes.c_int64, ctypes.c_int64]
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _dtype_code(a: np.ndarray, bf16: bool) -> int:
    if bf16:
        if a.dtype != np.uint16:
            raise TypeError("bf16 operands are passed as uint16 bit patterns")
        return BF16
    if a.dtype == np.float64:
        return F64
    if a.dtype == np.float32:
        return F32
    raise TypeError(f"unsupported dtype {a.dtype}")


def matmul(A: np.ndarray, B: np.ndarray, bf16: bool = False) -> np.ndarray:
    """fp64 ``A @ B`` by the triple loop.  A and B are 2-D, row-major (any row
    stride), of the same dtype: float64, float32, or uint16 holding bf16 bits
    (``bf16=True``)."""
    if A.ndim != 2 or B.ndim != 2 or A.shape[1] != B.shape[0]:
        raise ValueError("shapes do not form A[m,k] B[k,n]")
    code = _dtype_code(A, bf16)
    if _dtype_code(B, bf16) != code:
        raise TypeError("A and B must have the same dtype")
    A = _row_major(A)
    B = _row_major(B)
    m, k = A.shape
    n = B.shape[1]
    C = np.empty((m, n), dtype=np.float64)
    rc = _load().oracle_matmul(code,
                               A.ctypes.data, A.strides[0] // A.itemsize if m > 1 else max(k, 1),
                               B.ctypes.data, B.strides[0] // B.itemsize if k > 1 else max(n, 1),
                               C.ctypes.data, max(n, 1), m, k, n)
    if rc != 0:
        raise RuntimeError("oracle_matmul rejected its arguments")
    return C


def _row_major(X: np.ndarray) -> np.ndarray:
    """Rows must be contiguous; a row stride larger than the width is fine."""
    if X.shape[1] > 1 and X.strides[1] != X.itemsize:
        return np.ascontiguousarray(X)
    if X.shape[0] > 1 and (X.strides[0] % X.itemsize != 0 or X.strides[0] < X.shape[1] * X.itemsize):
        return np.ascontiguousarray(X)
    return X


def reduce_replicas(parts: Sequence[np.ndarray]) -> np.ndarray:
    """fp32 ``((parts[0] + parts[1]) + parts[2]) + ...`` of equally shaped 2-D
    fp32 arrays (Table 1, reduce_replicas; the order is this build's reading)."""
    parts = [np.ascontiguousarray(p, dtype=np.float32) for p in parts]
    rows, cols = parts[0].shape
    for p in parts:
        if p.shape != (rows, cols):
            raise ValueError("replica tiles differ in shape")
    out = np.empty((rows, cols), dtype=np.float32)
    n = len(parts)
    ptrs = (ctypes.c_void_p * n)(*[p.ctypes.data for p in parts])
    lds = (ctypes.c_int64 * n)(*[max(cols, 1)] * n)
    rc = _load().oracle_reduce_replicas(ptrs, lds, n, out.ctypes.data, max(cols, 1), rows, cols)
    if rc != 0:
        raise RuntimeError("oracle_reduce_replicas rejected its arguments")
    return out
