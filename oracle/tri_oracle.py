"""ctypes front end of the triangular-solve oracle (oracle/tri_oracle.c).

TEST INFRASTRUCTURE.  Only the tests, the smoke check and the benchmark's
cpu_baseline leg may import this module; the product package never does, and
this module imports nothing from the product package.

L is n x n (lower triangle and diagonal are read, nothing above), B and X are
n x nrhs, all row-major numpy arrays on the host.
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
        lib.tri_scalar_f64.argtypes = [ptr, ptr, ptr, i64, i64]
        lib.tri_scalar_f64.restype = ctypes.c_int
        lib.tri_tiled_bf16.argtypes = [ptr, ptr, ptr, ptr, i64, i64, i64]
        lib.tri_tiled_bf16.restype = ctypes.c_int
        _ready = True
    return lib


def tri_scalar(L, B) -> np.ndarray:
    """The scalar forward-substitution recurrence in fp64."""
    L = np.ascontiguousarray(L, dtype=np.float64)
    B = np.ascontiguousarray(B, dtype=np.float64)
    n, nrhs = B.shape
    if L.shape != (n, n):
        raise ValueError(f"shape mismatch: L {L.shape}, B {B.shape}")
    X = np.empty((n, nrhs), dtype=np.float64)
    _lib().tri_scalar_f64(L.ctypes.data, B.ctypes.data, X.ctypes.data, n, nrhs)
    return X


def tri_tiled(L_bits, B, nb: int):
    """The tiled recurrence in the library's arithmetic.  L_bits: uint16 bfloat16 bit patterns,
    B: float32.  Returns (X float32, Xh uint16 bfloat16 bit patterns of the rounded tiles)."""
    L_bits = np.ascontiguousarray(L_bits, dtype=np.uint16)
    B = np.ascontiguousarray(B, dtype=np.float32)
    n, nrhs = B.shape
    if L_bits.shape != (n, n):
        raise ValueError(f"shape mismatch: L {L_bits.shape}, B {B.shape}")
    X = np.empty((n, nrhs), dtype=np.float32)
    Xh = np.empty((n, nrhs), dtype=np.uint16)
    rc = _lib().tri_tiled_bf16(L_bits.ctypes.data, B.ctypes.data, X.ctypes.data, Xh.ctypes.data, n, nrhs, int(nb))
    if rc == -1:
        raise MemoryError("tri_tiled: allocation failed")
    if rc != 0:
        raise ValueError("tri_tiled: bad tile size")
    return X, Xh
