"""Pins of the attention oracle (oracle/attn_oracle.c): hand-worked values, closed forms and
invariants for the definition, and the tile recurrence against the definition for every tile size.

CPU only.  Mistakes planted in a copy of the recurrence must fail a hand-worked case.
"""
import math
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "attn_tiny_cases.txt")


@pytest.fixture(scope="module")
def attn():
    from oracle import attn_oracle
    return attn_oracle


def read_cases():
    cases, cur = [], None
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if not line:
            continue
        tok = line.split()
        if tok[0] == "case":
            cur = {"name": tok[1], "N": int(tok[2]), "M": int(tok[3]), "d": int(tok[4])}
            cases.append(cur)
        else:
            cur[tok[0]] = np.array([float(x) for x in tok[1:]], dtype=np.float64)
    for c in cases:
        c["Q"] = c["Q"].reshape(c["N"], c["d"])
        c["K"] = c["K"].reshape(c["M"], c["d"])
        c["V"] = c["V"].reshape(c["M"], c["d"])
        c["O"] = c["O"].reshape(c["N"], c["d"])
    return cases


def rand(N, M, d, seed, scale=1.0):
    rng = np.random.default_rng(seed)
    return rng.normal(size=(N, d)) * scale, rng.normal(size=(M, d)) * scale, rng.normal(size=(M, d))


@pytest.mark.parametrize("case", read_cases(), ids=lambda c: c["name"])
def test_hand_worked_cases(attn, case):
    O = attn.attention(case["Q"], case["K"], case["V"])
    assert np.allclose(O, case["O"], rtol=0, atol=2e-16 * max(1.0, np.abs(case["O"]).max()) * 4)
    for tile in (1, 2, 5):
        Or = attn.attention_recurrence(case["Q"], case["K"], case["V"], tile)
        assert np.allclose(Or, case["O"], rtol=0, atol=1e-15)


def test_planted_mistakes_fail_the_hand_worked_cases():
    """Plausible slips in the tile recurrence, each in a throw-away copy: every one misses the logistic
    or the three-key case (two or three tiles with a rising maximum)."""
    cases = {c["name"]: c for c in read_cases()}

    def run(c, tile=1, alpha=None, rescale_o=True, rescale_l=True, update_m=True, sub_max=True):
        Q, K, V = c["Q"], c["K"], c["V"]
        a = 1.0 / math.sqrt(c["d"]) if alpha is None else alpha
        O = np.zeros_like(c["O"])
        for i in range(c["N"]):
            m, l, o = -math.inf, 0.0, np.zeros(c["d"])
            for j0 in range(0, c["M"], tile):
                s = a * (K[j0:j0 + tile] @ Q[i])
                mh = max(m, s.max())
                keep = math.exp(m - mh)
                if rescale_l:
                    l *= keep
                if rescale_o:
                    o = o * keep
                p = np.exp(s - (mh if sub_max else 0.0))
                l += p.sum()
                o = o + p @ V[j0:j0 + tile]
                if update_m:
                    m = mh
            O[i] = o / l
        return O

    def ok(c, **kw):
        return np.allclose(run(c, **kw), c["O"], rtol=0, atol=1e-12)

    lo, th = cases["logistic"], cases["three_keys"]
    assert ok(lo) and ok(th) and ok(th, tile=2)                 # the copy itself is right
    assert not ok(lo, alpha=1.0)                                # scale 1/sqrt(d) forgotten
    assert not ok(lo, rescale_o=False)                          # old output not rescaled
    assert not ok(lo, rescale_l=False)                          # old sum not rescaled
    assert not ok(th, update_m=False)                           # running maximum never stored
    assert not ok(lo, sub_max=False)                            # exp of the raw score, rescaling kept


@pytest.mark.parametrize("N,M,d", [(1, 1, 1), (3, 5, 2), (17, 33, 8), (40, 130, 64), (9, 257, 128)])
def test_recurrence_equals_definition_for_every_tile_size(attn, N, M, d):
    Q, K, V = rand(N, M, d, seed=N + M + d, scale=1.5)
    ref = attn.attention(Q, K, V)
    for tile in (1, 3, 16, 64, M, M + 7):
        Or = attn.attention_recurrence(Q, K, V, tile)
        assert np.max(np.abs(Or - ref)) <= 1e-13 * max(1.0, np.abs(V).max())


def test_definition_against_a_direct_evaluation(attn):
    """exp / sum / weighted mean written with library calls on a small case (no maximum subtracted)."""
    Q, K, V = rand(6, 11, 4, seed=3)
    W = np.exp(Q @ K.T / 2.0)
    ref = (W / W.sum(axis=1, keepdims=True)) @ V
    assert np.max(np.abs(attn.attention(Q, K, V) - ref)) <= 1e-14


def test_invariants(attn):
    Q, K, V = rand(12, 70, 16, seed=8, scale=2.0)
    O = attn.attention(Q, K, V)
    # rows of O lie in the convex hull of the rows of V, coordinate by coordinate
    assert np.all(O <= V.max(axis=0) + 1e-12) and np.all(O >= V.min(axis=0) - 1e-12)
    # permuting the keys together with their values changes nothing
    perm = np.random.default_rng(1).permutation(70)
    assert np.max(np.abs(attn.attention(Q, K[perm], V[perm]) - O)) <= 1e-13
    # shifting every key by u adds Q_i.u to all scores of query i: softmax is unchanged
    u = np.random.default_rng(2).normal(size=16)
    assert np.max(np.abs(attn.attention(Q, K + u, V) - O)) <= 1e-12
    # a constant V comes back unchanged
    const = np.tile(np.arange(16.0), (70, 1))
    assert np.max(np.abs(attn.attention(Q, K, const) - np.arange(16.0))) <= 1e-13
    # queries are independent of one another
    assert np.array_equal(attn.attention(Q[3:5], K, V), O[3:5])


def test_dominant_key_and_large_scores(attn):
    """A key far ahead of the others takes all the weight; scores of several hundred must not overflow
    (the maximum is subtracted before exp)."""
    d = 16
    Q = np.zeros((1, d)); Q[0, 0] = 40.0
    K = np.zeros((5, d)); K[2, 0] = 40.0; K[1, 0] = 30.0
    V = np.arange(5 * d, dtype=np.float64).reshape(5, d)
    O = attn.attention(Q, K, V)
    assert np.all(np.isfinite(O))
    assert np.max(np.abs(O - V[2])) <= 100 * math.exp(-100.0) * np.abs(V).max() + 1e-12
    assert np.max(np.abs(attn.attention_recurrence(Q, K, V, 2) - O)) <= 1e-12


def test_empty_and_bad_arguments(attn):
    O = attn.attention(np.zeros((0, 4)), np.zeros((3, 4)), np.zeros((3, 4)))
    assert O.shape == (0, 4)
    with pytest.raises(ValueError):
        attn.attention_recurrence(np.zeros((2, 4)), np.zeros((3, 4)), np.zeros((3, 4)), 0)
    with pytest.raises(ValueError):
        attn.attention(np.zeros((2, 4)), np.zeros((3, 5)), np.zeros((3, 5)))
