"""Pins of the Cholesky oracle (oracle/chol_oracle.c) against things other than itself: hand-worked
factors, the fp64 library Cholesky, the identity L L^T = A, integer factors that are exact in every
arithmetic, closed forms, and the error the tiled bf16 recurrence may have against fp64.

CPU only.  Mistakes planted in a copy of the recurrence must fail the hand-worked case.
"""
import math
import os

import numpy as np
import pytest

from datagen import ws_inputs
from helpers import bits_to_f64

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "chol_tiny_cases.txt")


@pytest.fixture(scope="module")
def chol():
    from oracle import chol_oracle
    return chol_oracle


def read_cases():
    cases, cur = [], None
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if not line:
            continue
        tok = line.split()
        if tok[0] == "case":
            cur = {"name": tok[1], "n": int(tok[2]), "nb": int(tok[3])}
            cases.append(cur)
        else:
            v = [int(tok[i]) * 2.0 ** int(tok[i + 1]) for i in range(1, len(tok), 2)]
            cur[tok[0]] = np.array(v, dtype=np.float64).reshape(cur["n"], cur["n"])
    return cases


def spd(n, seed, upper=None):
    return ws_inputs.spd_f32(n, seed, 0, upper=upper).numpy()


def integer_factor(n, seed):
    """A lower-triangular factor of small integers (diagonal in {1, 2, 4}, a sparse {-1, 0, 1} pattern below)
    and A = L L^T, whose entries are integers far below 2^24: every arithmetic reproduces L exactly."""
    rng = np.random.default_rng(seed)
    L = np.tril(rng.integers(-1, 2, size=(n, n)) * (rng.random((n, n)) < 0.2), -1).astype(np.float64)
    L += np.diag(rng.choice([1.0, 2.0, 4.0], size=n))
    return L, L @ L.T


# ------------------------------------------------------------------ hand-worked values
@pytest.mark.parametrize("case", read_cases(), ids=lambda c: c["name"])
def test_hand_worked_cases(chol, case):
    if case["nb"] == 0:
        assert np.array_equal(chol.chol_scalar(case["A"]), case["L"])
        return
    L, Lh = chol.chol_tiled(case["A"].astype(np.float32), case["nb"])
    assert np.array_equal(L.astype(np.float64), case["L"])
    assert np.array_equal(bits_to_f64(Lh), case["LH"])


def test_one_tile_stays_in_fp32(chol):
    """The rounding case with a single tile: nothing is rounded to bfloat16 on the way, L_11 is the correctly
    rounded fp32 square root of fma(-x, x, 5), which is exactly representable."""
    x = np.float32(1 + 2.0 ** -9)
    A = np.array([[1, x], [x, 5]], dtype=np.float32)
    L, Lh = chol.chol_tiled(A, 2)
    t = 5.0 - float(x) * float(x)                       # 4 - 2^-8 - 2^-18: exact in fp64 and in fp32
    assert np.float32(t) == t
    assert L[1, 0] == x and L[1, 1] == np.sqrt(np.float32(t)) and L[1, 1] < 2.0
    assert bits_to_f64(Lh)[1, 0] == 1.0


def test_planted_mistakes_fail_the_hand_worked_case():
    """Plausible slips, each in a throw-away copy of the scalar recurrence: every one misses the 3 x 3 case."""
    case = {c["name"]: c for c in read_cases()}["three"]
    A, want = case["A"], case["L"]

    def run(sign=-1.0, root=True, divide_by="jj", swap=False, drop_first=False):
        n = A.shape[0]
        L = np.zeros((n, n))
        for i in range(n):
            for j in range(i + 1):
                t = A[j, i] if swap else A[i, j]
                for k in range(1 if drop_first else 0, j):
                    t += sign * L[i, k] * (L[k, j] if swap else L[j, k])
                if i == j:
                    L[i, i] = (math.sqrt(t) if t >= 0 else float("nan")) if root else t
                else:
                    L[i, j] = t / (L[j, j] if divide_by == "jj" else L[i - 1, i - 1])
        return L

    assert np.array_equal(run(), want)                                   # the copy itself is right
    assert not np.array_equal(run(sign=+1.0), want)                      # update added instead of subtracted
    assert not np.array_equal(run(root=False), want)                     # no square root on the diagonal
    assert not np.array_equal(run(divide_by="ii"), want)                 # divided by the wrong diagonal entry
    assert not np.array_equal(run(swap=True), want)                      # L_kj in place of L_jk
    assert not np.array_equal(run(drop_first=True), want)                # first term of the sums dropped


# ------------------------------------------------------------------ library routine, identities
@pytest.mark.parametrize("n", [1, 2, 3, 17, 64, 130])
def test_scalar_against_library_cholesky(chol, n):
    A = spd(n, 20 + n).astype(np.float64)
    L = chol.chol_scalar(A)
    ref = np.linalg.cholesky(A)
    assert np.max(np.abs(L - ref)) <= 1e-13
    assert np.array_equal(L, np.tril(L))
    assert np.max(np.abs(L @ L.T - A)) <= 1e-13 * np.abs(A).max()


@pytest.mark.parametrize("n,nb", [(1, 1), (5, 2), (64, 64), (96, 32), (130, 64), (200, 16), (150, 7)])
def test_tiled_within_bf16_rounding_of_fp64(chol, n, nb):
    """Each finished entry enters later sums with a relative error of 2^-9; the matrix is well conditioned
    (eigenvalues in about [1.5, 4.5], |L_ij| below 2.2), so the factor moves by a few times 2^-9 * max|L| at most,
    far less on average; with a single tile nothing is rounded and fp32 accuracy remains."""
    A = spd(n, 30 + n)
    ref = chol.chol_scalar(A.astype(np.float64))
    L, Lh = chol.chol_tiled(A, nb)
    err = np.abs(L.astype(np.float64) - ref)
    scale = np.abs(ref).max()
    if nb >= n:
        assert err.max() <= 64 * 2.0 ** -24 * scale
    else:
        assert err.max() <= 4 * 2.0 ** -9 * scale
        assert err.mean() <= 2.0 ** -12 * scale
    assert np.array_equal(L, np.tril(L)) and np.array_equal(Lh, np.tril(Lh))
    # Lh is L rounded to bfloat16: within half a unit of the 8th significant bit (2^-8 relative at worst)
    assert np.all(np.abs(bits_to_f64(Lh) - L) <= 2.0 ** -8 * np.abs(L) + 1e-45)
    # the factor reproduces A to bfloat16 accuracy
    assert np.max(np.abs(L.astype(np.float64) @ L.astype(np.float64).T - A)) <= 8 * 2.0 ** -9 * np.abs(A).max()


@pytest.mark.parametrize("n,nb", [(9, 1), (9, 2), (9, 4), (40, 16), (70, 64), (70, 100), (33, 5)])
def test_integer_factors_are_exact_for_every_tile_size(chol, n, nb):
    L0, A = integer_factor(n, 40 + n)
    assert np.abs(A).max() < 2 ** 20
    assert np.array_equal(chol.chol_scalar(A), L0)
    L, Lh = chol.chol_tiled(A.astype(np.float32), nb)
    assert np.array_equal(L.astype(np.float64), L0)
    assert np.array_equal(bits_to_f64(Lh), L0)


def test_closed_forms(chol):
    # diagonal A: L = sqrt(diag)
    d = np.array([1.0, 4.0, 9.0, 0.25, 16.0])
    assert np.array_equal(chol.chol_scalar(np.diag(d)), np.diag(np.sqrt(d)))
    L, Lh = chol.chol_tiled(np.diag(d).astype(np.float32), 2)
    assert np.array_equal(L, np.diag(np.sqrt(d)).astype(np.float32))
    # A = c^2 (I + 1 1^T) of order 2: L = c [[sqrt 2, 0], [1/sqrt 2, sqrt(3/2)]]
    L = chol.chol_scalar(np.array([[2.0, 1.0], [1.0, 2.0]]))
    assert np.allclose(L, [[math.sqrt(2), 0], [1 / math.sqrt(2), math.sqrt(1.5)]], rtol=1e-15, atol=0)
    # scaling A by 4 scales L by 2, exactly (powers of two commute with every rounding)
    A = spd(50, 3)
    L1, H1 = chol.chol_tiled(A, 16)
    L2, H2 = chol.chol_tiled(4 * A, 16)
    assert np.array_equal(L2, 2 * L1) and np.array_equal(bits_to_f64(H2), 2 * bits_to_f64(H1))


def test_upper_triangle_is_never_read(chol):
    A = spd(70, 5)
    B = spd(70, 5, upper=float("nan"))
    assert np.array_equal(np.tril(A), np.tril(B)) and np.isnan(B[0, 1])
    L1, H1 = chol.chol_tiled(A, 32)
    L2, H2 = chol.chol_tiled(B, 32)
    assert np.array_equal(L1, L2) and np.array_equal(H1, H2)
    assert np.array_equal(chol.chol_scalar(A.astype(np.float64)), chol.chol_scalar(B.astype(np.float64)))


def test_not_positive_definite_gives_nan_not_an_error(chol):
    A = np.array([[1.0, 2.0], [2.0, 1.0]], dtype=np.float32)
    L, Lh = chol.chol_tiled(A, 1)
    assert L[0, 0] == 1.0 and L[1, 0] == 2.0 and np.isnan(L[1, 1])


def test_empty_and_bad_arguments(chol):
    L, Lh = chol.chol_tiled(np.zeros((0, 0), dtype=np.float32), 4)
    assert L.shape == (0, 0)
    with pytest.raises(ValueError):
        chol.chol_tiled(np.eye(3, dtype=np.float32), 0)
    with pytest.raises(ValueError):
        chol.chol_scalar(np.zeros((2, 3)))
