"""Shared test helpers: conversions and the error metric.  No oracle code, no product code."""
from __future__ import annotations

import contextlib

import numpy as np
import torch


@contextlib.contextmanager
def forced(lib, name):
    """Inside the block the library uses the named kernel wherever it supports the problem (None: the dispatcher
    decides, whatever CYC_FORCE_KERNEL said when the library was loaded)."""
    assert lib.cyc_force_kernel(name or "") == 0, name
    try:
        yield
    finally:
        lib.cyc_force_kernel("")


def to_bf16_bits(x) -> np.ndarray:
    """float array -> uint16 bfloat16 bit patterns (round to nearest even, via torch)."""
    t = torch.as_tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def torch_bf16_to_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def rel_err(C, Cref, A64, B64) -> float:
    """max_ij |C_ij - Cref_ij| / sum_k |A_ik| |B_kj|  (denominator in fp64).

    Entries whose denominator is zero must match exactly."""
    C = np.asarray(C, dtype=np.float64)
    Cref = np.asarray(Cref, dtype=np.float64)
    den = np.abs(A64) @ np.abs(B64)
    diff = np.abs(C - Cref)
    zero = den == 0
    if np.any(diff[zero] != 0):
        return float("inf")
    if np.all(zero):
        return 0.0
    return float(np.max(diff[~zero] / den[~zero]))


# the tolerance the benchmark definition states for bf16 inputs with fp32 accumulation
BF16_TOL = 2e-2
