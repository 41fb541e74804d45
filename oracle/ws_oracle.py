"""ctypes front end of the CPU oracle (oracle/ws_oracle.c).

TEST INFRASTRUCTURE.  Only the tests, the smoke check and the benchmark's
cpu_baseline leg may import this module; the product package never does, and
this module imports nothing from the product package.

All functions take and return numpy arrays on the host:
  mode "i8":   A, B int8;  C int32
  mode "bf16": A, B uint16 holding bfloat16 bit patterns;  C float32
A is M x K, B is K x N, C is M x N, row-major (the paper's A_ik, B_kj, C_ij).
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.LIB if os.path.exists(_build.LIB) else _build.build()
        lib = ctypes.CDLL(path)
        i64, ptr = ctypes.c_int64, ctypes.c_void_p
        for sfx in ("i8", "bf16"):
            for name, res in (("ws_cells", ctypes.c_int), ("ws_wavefront", ctypes.c_int64),
                              ("ws_rowchain", ctypes.c_int)):
                fn = getattr(lib, f"{name}_{sfx}")
                fn.argtypes = [ptr, ptr, ptr, i64, i64, i64]
                fn.restype = res
        lib.ws_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


_IN = {"i8": np.int8, "bf16": np.uint16}
_OUT = {"i8": np.int32, "bf16": np.float32}


def _prep(A, B, mode):
    A = np.ascontiguousarray(A, dtype=_IN[mode])
    B = np.ascontiguousarray(B, dtype=_IN[mode])
    if A.ndim != 2 or B.ndim != 2 or A.shape[1] != B.shape[0]:
        raise ValueError(f"shape mismatch: A {A.shape}, B {B.shape}")
    M, K = A.shape
    N = B.shape[1]
    C = np.empty((M, N), dtype=_OUT[mode])
    return A, B, C, M, K, N


def _call(name, A, B, mode):
    A, B, C, M, K, N = _prep(A, B, mode)
    fn = getattr(_load(), f"{name}_{mode}")
    rc = fn(A.ctypes.data, B.ctypes.data, C.ctypes.data, M, K, N)
    return C, rc


def ws_cells(A, B, mode):
    """Sequential literal cell grid (nine per-cell programs)."""
    C, rc = _call("ws_cells", A, B, mode)
    if rc != 0:
        raise MemoryError("ws_cells: allocation failed")
    return C


def ws_wavefront(A, B, mode):
    """Clocked grid with unit-latency links.  Returns (C, active_ticks).

    Raises if any operand reached a cell at a tick other than i+j+k."""
    C, rc = _call("ws_wavefront", A, B, mode)
    if rc == -1:
        raise MemoryError("ws_wavefront: allocation failed")
    if rc < -1:
        raise AssertionError(f"ws_wavefront: {-2 - rc} operands arrived at the wrong tick")
    return C, int(rc)


def ws_rowchain(A, B, mode):
    """k-ordered accumulator chain per (i,j), rows spread over host cores."""
    C, _ = _call("ws_rowchain", A, B, mode)
    return C


def threads() -> int:
    return int(_load().ws_oracle_threads())


def bf16_bits(t) -> np.ndarray:
    """torch.bfloat16 CPU tensor -> uint16 numpy array of its bit patterns."""
    import torch
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns -> their exact values as float64."""
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
