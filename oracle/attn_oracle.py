"""ctypes front end of the attention oracle (oracle/attn_oracle.c).

TEST INFRASTRUCTURE.  Only the tests, the smoke check and the benchmark's
cpu_baseline leg may import this module; the product package never does, and
this module imports nothing from the product package.

Q is N x d, K and V are M x d, O is N x d; row-major numpy float64 arrays on the host.
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
        lib.attn_definition_f64.argtypes = [ptr, ptr, ptr, ptr, i64, i64, i64]
        lib.attn_definition_f64.restype = ctypes.c_int
        lib.attn_recurrence_f64.argtypes = [ptr, ptr, ptr, ptr, i64, i64, i64, i64]
        lib.attn_recurrence_f64.restype = ctypes.c_int
        _ready = True
    return lib


def _prep(Q, K, V):
    Q = np.ascontiguousarray(Q, dtype=np.float64)
    K = np.ascontiguousarray(K, dtype=np.float64)
    V = np.ascontiguousarray(V, dtype=np.float64)
    if Q.ndim != 2 or K.ndim != 2 or K.shape != V.shape or Q.shape[1] != K.shape[1]:
        raise ValueError(f"shape mismatch: Q {Q.shape}, K {K.shape}, V {V.shape}")
    return Q, K, V, np.empty(Q.shape, dtype=np.float64)


def attention(Q, K, V) -> np.ndarray:
    """O = softmax(Q K^T / sqrt(d)) V, the definition, in fp64."""
    Q, K, V, O = _prep(Q, K, V)
    rc = _lib().attn_definition_f64(Q.ctypes.data, K.ctypes.data, V.ctypes.data, O.ctypes.data, Q.shape[0], K.shape[0],
                                    Q.shape[1])
    if rc != 0:
        raise MemoryError("attention: allocation failed")
    return O


def attention_recurrence(Q, K, V, tile: int) -> np.ndarray:
    """The tile recurrence (running maximum, sum and output per query) in fp64, key tiles of `tile` keys."""
    Q, K, V, O = _prep(Q, K, V)
    rc = _lib().attn_recurrence_f64(Q.ctypes.data, K.ctypes.data, V.ctypes.data, O.ctypes.data, Q.shape[0], K.shape[0],
                                    Q.shape[1], int(tile))
    if rc == -1:
        raise MemoryError("attention_recurrence: allocation failed")
    if rc != 0:
        raise ValueError("attention_recurrence: bad tile size")
    return O
