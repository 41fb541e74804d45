"""ctypes front end of the Cholesky oracle (oracle/chol_oracle.c).

TEST INFRASTRUCTURE.  Only the tests, the smoke check and the benchmark's
cpu_baseline leg may import this module; the product package never does, and
this module imports nothing from the product package.

A is n x n symmetric positive definite (only its lower triangle is read), L is
its lower-triangular factor, A = L L^T; row-major numpy arrays on the host.
"""
from __future__ import annotations

import ctypes

import numpy as np

from . import ws_oracle

_ready = False


def _lib():
    global _ready
    lib = ws_oracle._load()
    if not _ready:
        i64, ptr = ctypes.c_int64, ctypes.c_void_p
        lib.chol_scalar_f64.argtypes = [ptr, ptr, i64]
        lib.chol_scalar_f64.restype = ctypes.c_int
        lib.chol_tiled_bf16.argtypes = [ptr, ptr, ptr, i64, i64]
        lib.chol_tiled_bf16.restype = ctypes.c_int
        _ready = True
    return lib


def chol_scalar(A) -> np.ndarray:
    """The scalar Cholesky recurrence in fp64."""
    A = np.ascontiguousarray(A, dtype=np.float64)
    n = A.shape[0]
    if A.shape != (n, n):
        raise ValueError(f"A must be square, got {A.shape}")
    L = np.empty((n, n), dtype=np.float64)
    _lib().chol_scalar_f64(A.ctypes.data, L.ctypes.data, n)
    return L


def chol_tiled(A, nb: int):
    """The tiled recurrence in the library's arithmetic.  A: float32.  Returns (L float32, Lh uint16
    bfloat16 bit patterns of the rounded tiles), both lower triangular with zeros above the diagonal."""
    A = np.ascontiguousarray(A, dtype=np.float32)
    n = A.shape[0]
    if A.shape != (n, n):
        raise ValueError(f"A must be square, got {A.shape}")
    L = np.empty((n, n), dtype=np.float32)
    Lh = np.empty((n, n), dtype=np.uint16)
    rc = _lib().chol_tiled_bf16(A.ctypes.data, L.ctypes.data, Lh.ctypes.data, n, int(nb))
    if rc == -1:
        raise MemoryError("chol_tiled: allocation failed")
    if rc != 0:
        raise ValueError("chol_tiled: bad tile size")
    return L, Lh
