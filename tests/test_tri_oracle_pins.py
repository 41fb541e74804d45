"""Pins of the triangular-solve oracle (oracle/tri_oracle.c) against things other than itself:
hand-worked values, a library fp64 triangular solve, closed forms, integer systems that are exact
in every arithmetic, and the error the tiled bf16 recurrence may have against fp64.

CPU only.  Mistakes planted in a copy of the recurrence must fail the hand-worked case.
"""
import math
import os

import numpy as np
import pytest
import scipy.linalg
import torch

from datagen import ws_inputs
from helpers import bits_to_f64, to_bf16_bits, torch_bf16_to_bits

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "tri_tiny_cases.txt")


@pytest.fixture(scope="module")
def tri():
    from oracle import tri_oracle
    return tri_oracle


def read_cases():
    cases, cur = [], None
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if not line:
            continue
        tok = line.split()
        if tok[0] == "case":
            cur = {"name": tok[1], "n": int(tok[2]), "nrhs": int(tok[3]), "nb": int(tok[4])}
            cases.append(cur)
        else:
            v = [int(tok[i]) * 2.0 ** int(tok[i + 1]) for i in range(1, len(tok), 2)]
            cur[tok[0]] = np.array(v, dtype=np.float64)
    return cases


def well_conditioned(n, nrhs, seed):
    """(L as bf16 bits, L as fp64, B fp32) from the seeded recipe of the workloads."""
    L = ws_inputs.tri_lower_bf16(n, seed, 0)
    B = ws_inputs.normal_f32((n, nrhs), 1.0, seed, 1)
    bits = torch_bf16_to_bits(L)
    return bits, bits_to_f64(bits), B.numpy()


# ------------------------------------------------------------------ hand-worked values
@pytest.mark.parametrize("case", read_cases(), ids=lambda c: c["name"])
def test_hand_worked_cases(tri, case):
    n, nrhs, nb = case["n"], case["nrhs"], case["nb"]
    L = case["L"].reshape(n, n)
    B = case["B"].reshape(n, nrhs)
    if nb == 0:
        assert np.array_equal(tri.tri_scalar(L, B), case["X"].reshape(n, nrhs))
        return
    X, Xh = tri.tri_tiled(to_bf16_bits(L), B.astype(np.float32), nb)
    assert np.array_equal(X.astype(np.float64), case["X"].reshape(n, nrhs))
    assert np.array_equal(bits_to_f64(Xh), case["XH"].reshape(n, nrhs))


def test_planted_mistakes_fail_the_hand_worked_case():
    """Plausible slips in the recurrence, each in a throw-away copy of it: none reproduces the
    hand-worked 3 x 3 solution."""
    case = [c for c in read_cases() if c["name"] == "int3"][0]
    L = case["L"].reshape(3, 3)
    B = case["B"].reshape(3, 2)
    want = case["X"].reshape(3, 2)

    def solve(sign=-1.0, upto=lambda i: i, transpose=False, divide=True, diag=lambda L, i: L[i, i]):
        M = L.T if transpose else L
        X = np.zeros_like(B)
        for i in range(3):
            t = B[i].copy()
            for j in range(upto(i)):
                t += sign * M[i, j] * X[j]
            X[i] = t / diag(M, i) if divide else t
        return X

    assert np.array_equal(solve(), want)                                   # the copy itself is right
    assert not np.array_equal(solve(sign=+1.0), want)                      # added instead of subtracted
    assert not np.array_equal(solve(upto=lambda i: max(i - 1, 0)), want)   # last term dropped
    assert not np.array_equal(solve(transpose=True), want)                 # L_ji for L_ij
    assert not np.array_equal(solve(divide=False), want)                   # division forgotten
    assert not np.array_equal(solve(diag=lambda L, i: L[0, 0]), want)      # wrong diagonal entry


# ------------------------------------------------------------------ the scalar recurrence
@pytest.mark.parametrize("n,nrhs", [(1, 1), (2, 3), (7, 5), (33, 4), (200, 17)])
def test_scalar_matches_library_solve(tri, n, nrhs):
    _, L, B = well_conditioned(n, nrhs, seed=100 + n)
    X = tri.tri_scalar(L, B)
    ref = scipy.linalg.solve_triangular(L, B.astype(np.float64), lower=True)
    assert np.max(np.abs(X - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))
    # and it solves the system
    assert np.max(np.abs(np.tril(L) @ X - B)) <= 1e-12 * n * max(1.0, np.max(np.abs(X)))


# ------------------------------------------------------------------ the tiled bf16 / fp32 recurrence
def skeel(L):
    """|| |L^-1| |L| ||_inf, the condition number that governs forward substitution."""
    Linv = scipy.linalg.solve_triangular(L, np.eye(L.shape[0]), lower=True)
    return float(np.max(np.sum(np.abs(Linv) @ np.abs(np.tril(L)), axis=1)))


@pytest.mark.parametrize("n,nrhs,nb", [(8, 3, 2), (64, 9, 16), (200, 8, 32), (200, 8, 128), (513, 5, 64),
                                       (96, 33, 1)])
def test_tiled_is_close_to_fp64(tri, n, nrhs, nb):
    """Against the fp64 recurrence on the same (bf16-valued) L: the only errors are the bf16
    rounding of X where it enters the GEMMs (relative 2^-9 per element) and fp32 rounding."""
    bits, L, B = well_conditioned(n, nrhs, seed=200 + n + nb)
    X, Xh = tri.tri_tiled(bits, B, nb)
    ref = tri.tri_scalar(L, B)
    scale = np.max(np.abs(ref))
    err = np.max(np.abs(X - ref)) / scale
    assert err <= 2.0 ** -9 * skeel(L) * 2, err
    assert err >= 2.0 ** -14, "suspiciously exact: X must have been rounded to bfloat16 on its way"
    # the published bf16 values are the nearest bf16 to X
    assert np.array_equal(Xh, to_bf16_bits(X))


@pytest.mark.parametrize("n,nrhs", [(5, 2), (64, 7), (200, 8)])
def test_one_tile_is_the_scalar_recurrence_in_fp32(tri, n, nrhs):
    """With nb >= n nothing is rounded to bf16 on the way: the error against fp64 drops to fp32 level."""
    bits, L, B = well_conditioned(n, nrhs, seed=300 + n)
    X, _ = tri.tri_tiled(bits, B, n + 3)
    ref = tri.tri_scalar(L, B)
    err = np.max(np.abs(X - ref)) / np.max(np.abs(ref))
    assert err <= n * 2.0 ** -23 * skeel(L)


def integer_system(n, nrhs, seed, density=0.2):
    """L with diagonal in {1, 2, -1, 4, -2} and sparse entries in {-1, 0, 1} below it, X small
    integers, B = L X computed exactly: every intermediate of any forward substitution is an
    integer far below 2^24, every X is exact in bfloat16, every division is by a power of two."""
    rng = np.random.default_rng(seed)
    L = np.tril(rng.integers(-1, 2, size=(n, n)) * (rng.random((n, n)) < density), -1).astype(np.int64)
    L[np.arange(n), np.arange(n)] = rng.choice([1, 2, -1, 4, -2], size=n)
    X = rng.integers(-8, 9, size=(n, nrhs)).astype(np.int64)
    B = L @ X
    assert np.max(np.abs(B)) < 2 ** 20
    return L, X, B


@pytest.mark.parametrize("nb", [1, 3, 16, 64, 1000])
def test_integer_systems_are_exact_for_every_tile_size(tri, nb):
    L, Xtrue, B = integer_system(150, 11, seed=7)
    X, Xh = tri.tri_tiled(to_bf16_bits(L), B.astype(np.float32), nb)
    assert np.array_equal(X, Xtrue.astype(np.float32))
    assert np.array_equal(bits_to_f64(Xh), Xtrue.astype(np.float64))
    assert np.array_equal(tri.tri_scalar(L.astype(np.float64), B.astype(np.float64)), Xtrue.astype(np.float64))


def test_identity_and_diagonal_weights(tri):
    n, nrhs = 70, 6
    B = ws_inputs.normal_f32((n, nrhs), 1.0, 5, 0).numpy()
    X, Xh = tri.tri_tiled(to_bf16_bits(np.eye(n)), B, 16)
    assert np.array_equal(X, B) and np.array_equal(Xh, to_bf16_bits(B))
    d = 2.0 ** (np.arange(n) % 7 - 3)
    X, _ = tri.tri_tiled(to_bf16_bits(np.diag(d)), B, 16)
    assert np.array_equal(X, (B / d[:, None]).astype(np.float32))       # exact: powers of two


def test_columns_are_independent_and_upper_triangle_is_never_read(tri):
    n, nrhs, nb = 100, 40, 32
    bits, L, B = well_conditioned(n, nrhs, seed=9)
    X, Xh = tri.tri_tiled(bits, B, nb)
    cols = [3, 17, 39]
    Xs, Xhs = tri.tri_tiled(bits, B[:, cols], nb)
    assert np.array_equal(Xs, X[:, cols]) and np.array_equal(Xhs, Xh[:, cols])
    poisoned = bits.copy()
    poisoned[np.triu_indices(n, 1)] = 0x7FC0                            # NaN above the diagonal
    Xp, _ = tri.tri_tiled(poisoned, B, nb)
    assert np.array_equal(Xp, X)
    Lp = L.copy()
    Lp[np.triu_indices(n, 1)] = np.nan
    assert np.array_equal(tri.tri_scalar(Lp, B), tri.tri_scalar(L, B))


def test_ragged_last_tile_and_empty_inputs(tri):
    L, Xtrue, B = integer_system(37, 3, seed=11)
    for nb in (5, 36, 37, 38):
        X, _ = tri.tri_tiled(to_bf16_bits(L), B.astype(np.float32), nb)
        assert np.array_equal(X, Xtrue.astype(np.float32))
    X, Xh = tri.tri_tiled(np.zeros((0, 0), np.uint16), np.zeros((0, 4), np.float32), 8)
    assert X.shape == (0, 4) and Xh.shape == (0, 4)
    with pytest.raises(ValueError):
        tri.tri_tiled(to_bf16_bits(np.eye(4)), np.zeros((4, 1), np.float32), 0)
