"""Pins of the CPU oracle to things other than itself (CPU only).

Each test checks oracle/ws_oracle.c against something the paper or the
mathematics fixes: hand-worked values, a library matmul in wider precision,
closed forms (identity weights, rank-1, all-ones, one-hot), the sum identity,
and the timing invariant t = i+j+k of the paper's Timing section.
"""
import itertools
import os

import numpy as np
import pytest
import torch

from datagen import ws_inputs
from helpers import bits_to_f64, to_bf16_bits, torch_bf16_to_bits

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "ws_tiny_cases.txt")
FORMS = ("ws_cells", "ws_rowchain", "ws_wavefront")


def run(oracle, form, A, B, mode):
    out = getattr(oracle, form)(A, B, mode)
    return out[0] if form == "ws_wavefront" else out


def rand_inputs(mode, M, K, N, seed):
    if mode == "i8":
        A = ws_inputs.uniform_int((M, K), 127, seed, 0).numpy()
        B = ws_inputs.uniform_int((K, N), 127, seed, 1).numpy()
    else:
        A = torch_bf16_to_bits(ws_inputs.normal_bf16((M, K), 1.0, seed, 0))
        B = torch_bf16_to_bits(ws_inputs.normal_bf16((K, N), 1.0, seed, 1))
    return A, B


def widen(X, mode):
    return X.astype(np.int64) if mode == "i8" else bits_to_f64(X)


# ---------------------------------------------------------------- golden file
def _parse_golden():
    cases, cur = [], None
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if not line:
            continue
        tok = line.split()
        if tok[0] == "case":
            cur = {"name": tok[1], "mode": tok[2], "shape": tuple(map(int, tok[3:6]))}
            cases.append(cur)
        else:
            vals = list(map(int, tok[1:]))
            if cur["mode"] == "bf16":
                vals = [p * 2.0 ** e for p, e in zip(vals[0::2], vals[1::2])]
            cur[tok[0]] = vals
    return cases


@pytest.mark.parametrize("case", _parse_golden(), ids=lambda c: c["name"])
@pytest.mark.parametrize("form", FORMS)
def test_hand_worked_cases(oracle, case, form):
    M, K, N = case["shape"]
    mode = case["mode"]
    if mode == "i8":
        A = np.array(case["A"], dtype=np.int8).reshape(M, K)
        B = np.array(case["B"], dtype=np.int8).reshape(K, N)
        want = np.array(case["C"], dtype=np.int32).reshape(M, N)
    else:
        A = to_bf16_bits(np.array(case["A"]).reshape(M, K))
        B = to_bf16_bits(np.array(case["B"]).reshape(K, N))
        assert np.array_equal(bits_to_f64(A).ravel(), case["A"])   # values are exact in bf16
        want = np.array(case["C"], dtype=np.float32).reshape(M, N)
    got = run(oracle, form, A, B, mode)
    assert got.tobytes() == want.tobytes()


def test_planted_mistakes_fail_a_hand_worked_case():
    """Plausible slips in the chain, each in a throw-away copy of it (fp32 accumulator, k ascending): every one of
    them gets at least one hand-worked case wrong, so the golden file would catch the same slip in the oracle."""
    cases = {c["name"]: c for c in _parse_golden()}

    def chain(case, order=lambda K: range(K), b_index=lambda B, k, j: B[k][j], first=0, widen=np.float32):
        M, K, N = case["shape"]
        A = np.array(case["A"], dtype=np.float64).reshape(M, K)
        B = np.array(case["B"], dtype=np.float64).reshape(K, N)
        C = np.zeros((M, N), dtype=np.float64)
        for i in range(M):
            for j in range(N):
                acc = widen(0)
                for k in order(K):
                    if k >= first:
                        acc = widen(acc + widen(A[i][k] * b_index(B, k, j)))
                C[i][j] = acc
        return C.ravel().tolist()

    def wrong_somewhere(**slip):
        return any(chain(c, **slip) != [float(v) for v in c["C"]] for c in cases.values()
                   if not ("b_index" in slip and c["shape"][1] != c["shape"][2]))     # B^T needs a square B

    assert not wrong_somewhere()                                               # the copy itself is right on every case
    assert wrong_somewhere(order=lambda K: range(K - 1, -1, -1))               # k descending (order1x3x1)
    assert wrong_somewhere(b_index=lambda B, k, j: B[j][k])                    # B_jk for B_kj (int2x2)
    assert wrong_somewhere(first=1)                                            # first term of the chain dropped
    assert wrong_somewhere(widen=np.float64)                                   # accumulator wider than fp32 (order1x3x1)


# ------------------------------------------- library matmul in wider precision
SMALL = list(itertools.product((1, 2, 3, 5, 8), repeat=3))
ODD = [(33, 17, 9), (9, 33, 17), (17, 9, 33), (31, 32, 33), (2, 64, 3)]


@pytest.mark.parametrize("form", FORMS)
def test_int_equals_int64_matmul(oracle, form):
    for n, (M, K, N) in enumerate(SMALL + ODD):
        A, B = rand_inputs("i8", M, K, N, seed=100 + n)
        want = A.astype(np.int64) @ B.astype(np.int64)
        got = run(oracle, form, A, B, "i8")
        assert got.dtype == np.int32 and got.shape == (M, N)
        assert np.array_equal(got.astype(np.int64), want), (M, K, N)


@pytest.mark.parametrize("form", FORMS)
def test_bf16_within_fp32_chain_bound_of_fp64_matmul(oracle, form):
    """|chain - exact| <= gamma_K * sum_k |a||b| with gamma_K = K u / (1 - K u), u = 2^-24."""
    u = 2.0 ** -24
    for n, (M, K, N) in enumerate(SMALL + ODD):
        A, B = rand_inputs("bf16", M, K, N, seed=200 + n)
        A64, B64 = bits_to_f64(A), bits_to_f64(B)
        exact = A64 @ B64
        bound = (K * u / (1 - K * u)) * (np.abs(A64) @ np.abs(B64))
        got = run(oracle, form, A, B, "bf16").astype(np.float64)
        assert np.all(np.abs(got - exact) <= bound + 1e-300), (M, K, N)


def test_bf16_long_chain_against_fp64(oracle):
    """K = 4096: the chain's error stays far below the bound and is not zero
    (an fp64 accumulator rounded at the end would be within 2^-24 relative)."""
    A, B = rand_inputs("bf16", 8, 4096, 8, seed=7)
    A64, B64 = bits_to_f64(A), bits_to_f64(B)
    exact = A64 @ B64
    got = oracle.ws_rowchain(A, B, "bf16").astype(np.float64)
    den = np.abs(A64) @ np.abs(B64)
    err = np.max(np.abs(got - exact) / den)
    assert err <= 4096 * 2.0 ** -24
    assert err > 2.0 ** -30


# ----------------------------------------------------- the three forms agree
@pytest.mark.parametrize("mode", ("i8", "bf16"))
def test_forms_bit_identical(oracle, mode):
    for n, (M, K, N) in enumerate(SMALL[::3] + ODD + [(40, 70, 24)]):
        A, B = rand_inputs(mode, M, K, N, seed=300 + n)
        ref = oracle.ws_cells(A, B, mode)
        assert oracle.ws_rowchain(A, B, mode).tobytes() == ref.tobytes(), (M, K, N)
        assert oracle.ws_wavefront(A, B, mode)[0].tobytes() == ref.tobytes(), (M, K, N)


# ------------------------------------------------------------------ timing
@pytest.mark.parametrize("mode", ("i8", "bf16"))
def test_wavefront_tick_count(oracle, mode):
    """Every operand meets at tick i+j+k (checked inside ws_wavefront, which raises
    otherwise) and the grid is busy for exactly M+K+N-2 ticks."""
    for n, (M, K, N) in enumerate(SMALL + ODD):
        A, B = rand_inputs(mode, M, K, N, seed=400 + n)
        _, ticks = oracle.ws_wavefront(A, B, mode)
        assert ticks == M + K + N - 2, (M, K, N)


# -------------------------------------------------------------- closed forms
def as_mode(X, mode):
    X = np.asarray(X)
    return X.astype(np.int8) if mode == "i8" else to_bf16_bits(X.astype(np.float32))


def out_values(C):
    return C.astype(np.float64)


@pytest.mark.parametrize("mode", ("i8", "bf16"))
@pytest.mark.parametrize("form", FORMS)
def test_identity_weights_pass_B_through(oracle, mode, form):
    for K, N in ((1, 1), (5, 3), (16, 7), (33, 40)):
        _, B = rand_inputs(mode, K, K, N, seed=500 + K)
        A = as_mode(np.eye(K), mode)
        got = run(oracle, form, A, B, mode)
        assert np.array_equal(out_values(got), widen(B, mode).astype(np.float64))


@pytest.mark.parametrize("mode", ("i8", "bf16"))
@pytest.mark.parametrize("form", FORMS)
def test_rank_one(oracle, mode, form):
    rng = np.random.default_rng(11)
    for M, K, N in ((4, 1, 6), (7, 5, 3), (12, 9, 10)):
        u, v = rng.integers(-5, 6, M), rng.integers(-5, 6, N)
        w, z = rng.integers(-3, 4, K), rng.integers(-3, 4, K)
        A = as_mode(np.outer(u, w), mode)          # A = u w^T
        B = as_mode(np.outer(z, v), mode)          # B = z v^T
        want = int(w @ z) * np.outer(u, v)         # C = (w.z) u v^T
        got = run(oracle, form, A, B, mode)
        assert np.array_equal(out_values(got), want.astype(np.float64))


@pytest.mark.parametrize("mode", ("i8", "bf16"))
def test_all_ones_gives_K(oracle, mode):
    for form, shapes in (("ws_cells", ((3, 7, 2), (9, 100, 4))),
                         ("ws_wavefront", ((3, 7, 2), (4, 50, 3))),
                         ("ws_rowchain", ((3, 7, 2), (5, 8192, 3), (2, 20000, 2)))):
        for M, K, N in shapes:
            A, B = as_mode(np.ones((M, K)), mode), as_mode(np.ones((K, N)), mode)
            got = run(oracle, form, A, B, mode)
            assert np.all(out_values(got) == K), (form, M, K, N)


@pytest.mark.parametrize("mode", ("i8", "bf16"))
@pytest.mark.parametrize("form", FORMS)
def test_one_hot_probes(oracle, mode, form):
    """A = e_p e_q^T, B = e_q' e_r^T  =>  C = [q == q'] e_p e_r^T."""
    M, K, N = 5, 6, 4
    for p, q, q2, r in ((0, 0, 0, 0), (4, 5, 5, 3), (2, 3, 3, 1), (2, 3, 4, 1), (0, 5, 5, 3), (4, 0, 0, 0)):
        A = np.zeros((M, K)); A[p, q] = 3
        B = np.zeros((K, N)); B[q2, r] = -2
        want = np.zeros((M, N)); want[p, r] = -6 if q == q2 else 0
        got = run(oracle, form, as_mode(A, mode), as_mode(B, mode), mode)
        assert np.array_equal(out_values(got), want)


def test_int_wraps_mod_2_32(oracle):
    """Partial sums are int32 with two's-complement wrap: K = 2^17+8 products of (-128)(-128) = 2^14
    sum to 2^31 + 2^17, which wraps to -2^31 + 2^17."""
    K = (1 << 17) + 8
    A = np.full((1, K), -128, dtype=np.int8)
    B = np.full((K, 1), -128, dtype=np.int8)
    got = oracle.ws_rowchain(A, B, "i8")
    assert int(got[0, 0]) == -(1 << 31) + (1 << 17)


@pytest.mark.parametrize("mode", ("i8", "bf16"))
def test_sum_identity(oracle, mode):
    """sum_ij C_ij = sum_k (sum_i A_ik)(sum_j B_kj); exact for ints, and for small-integer bf16 data."""
    M, K, N = 37, 129, 21
    if mode == "i8":
        A, B = rand_inputs("i8", M, K, N, seed=9)
    else:
        A = torch_bf16_to_bits(ws_inputs.small_int_bf16((M, K), 8, 9, 0))
        B = torch_bf16_to_bits(ws_inputs.small_int_bf16((K, N), 8, 9, 1))
    C = oracle.ws_rowchain(A, B, mode)
    lhs = int(out_values(C).sum())
    rhs = int((widen(A, mode).sum(axis=0) * widen(B, mode).sum(axis=1)).sum())
    assert lhs == rhs


def test_degenerate_extents(oracle):
    for mode in ("i8", "bf16"):
        for form in FORMS:
            A = np.zeros((3, 0), dtype=np.int8 if mode == "i8" else np.uint16)
            B = np.zeros((0, 4), dtype=A.dtype)
            got = run(oracle, form, A, B, mode)
            assert got.shape == (3, 4) and np.all(got == 0)     # empty chain = its initial value
            got = run(oracle, form, np.zeros((0, 5), A.dtype), np.zeros((5, 4), A.dtype), mode)
            assert got.shape == (0, 4)


def test_small_int_bf16_is_order_independent(oracle):
    """With integer data of magnitude <= 8, every partial sum is an integer below 2^24, so the
    fp32 chain equals the exact integer product (the property GPU parity tests rely on to compare
    bit for bit at any size)."""
    M, K, N = 16, 2048, 16
    A = ws_inputs.small_int_bf16((M, K), 8, 21, 0)
    B = ws_inputs.small_int_bf16((K, N), 8, 21, 1)
    want = A.to(torch.int64) @ B.to(torch.int64)
    got = oracle.ws_rowchain(torch_bf16_to_bits(A), torch_bf16_to_bits(B), "bf16")
    assert np.array_equal(got.astype(np.int64), want.numpy())
