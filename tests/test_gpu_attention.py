"""GPU parity of the attention recurrence (cyc_recurrence_attention, through the C ABI) against the
CPU oracle (oracle/attn_oracle.c: the softmax definition in fp64 on the same bfloat16 inputs).

Tolerance.  The library keeps scores, maxima, sums and outputs in fp32 and rounds the exponentials to
bfloat16 (relative 2^-9) before the product with V; the running sum takes them unrounded.  O_i is a
weighted mean of the rows of V, so an element is off by at most about 2 * 2^-9 * max|V| (numerator and
denominator weights each within 2^-9), plus fp32 rounding and the hardware exp2 (a few 2^-22).  The
tests demand 2^-7 * max|V| as a hard bound on every element and 2^-10 * max|V| on the mean error
(roundings of different keys cancel), which is far below what a wrong tile, mask or rescale produces.
"""
import os

import numpy as np
import pytest
import torch

from datagen import ws_inputs
from helpers import bits_to_f64, torch_bf16_to_bits

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def lib():
    import paper_2511_09987_amd as pkg
    assert os.path.exists(pkg.lib_path()), "libcyclotron_mm.so must be built in-tree"
    return pkg


@pytest.fixture(scope="module")
def attn():
    from oracle import attn_oracle
    return attn_oracle


def f64(t):
    return bits_to_f64(torch_bf16_to_bits(t))


def check(O, ref, V64):
    O = O.cpu().numpy().astype(np.float64)
    vmax = np.abs(V64).max()
    assert np.all(np.isfinite(O))
    err = np.abs(O - ref)
    assert err.max() <= 2.0 ** -7 * vmax, f"max error {err.max():.3e} vs max|V| {vmax:.3e}"
    assert err.mean() <= 2.0 ** -10 * vmax, f"mean error {err.mean():.3e}"


SHAPES = [(1, 256, 256, 128), (1, 64, 64, 64), (1, 100, 130, 128), (1, 1, 1, 64), (1, 300, 1000, 64),
          (1, 257, 65, 128), (3, 128, 192, 128), (2, 70, 63, 64), (1, 512, 64, 128), (1, 16, 2048, 128)]


@pytest.mark.parametrize("batch,N,M,d", SHAPES)
def test_against_oracle(lib, attn, batch, N, M, d):
    Q = ws_inputs.normal_bf16((batch, N, d), 1.0, 10 + N, 0, DEV)
    K = ws_inputs.normal_bf16((batch, M, d), 1.0, 10 + N, 1, DEV)
    V = ws_inputs.normal_bf16((batch, M, d), 1.0, 10 + N, 2, DEV)
    O = lib.recurrence_attention(Q, K, V)
    torch.cuda.synchronize()
    for b in range(batch):
        ref = attn.attention(f64(Q[b]), f64(K[b]), f64(V[b]))
        check(O[b], ref, f64(V[b]))


def test_seeded_sweep_of_shapes(lib, attn):
    """Sixteen shapes drawn from a fixed seed: query and key counts from 1 to about 600 (ragged ends of both kinds,
    several key tiles, a last tile of any length), both head dimensions, one to three batch elements."""
    rng = np.random.default_rng(987)
    for i in range(16):
        batch, N, M, d = int(rng.integers(1, 4)), int(rng.integers(1, 600)), int(rng.integers(1, 600)), (64, 128)[i % 2]
        Q = ws_inputs.normal_bf16((batch, N, d), 1.5, 300 + i, 0, DEV)
        K = ws_inputs.normal_bf16((batch, M, d), 1.5, 300 + i, 1, DEV)
        V = ws_inputs.normal_bf16((batch, M, d), 1.0, 300 + i, 2, DEV)
        O = lib.recurrence_attention(Q, K, V)
        torch.cuda.synchronize()
        for b in range(batch):
            check(O[b], attn.attention(f64(Q[b]), f64(K[b]), f64(V[b])), f64(V[b]))


def test_sharp_scores(lib, attn):
    """Scores spread over +-30: the running maximum moves from tile to tile and old contributions are
    rescaled by tiny factors; nothing may overflow."""
    N, M, d = 192, 700, 128
    Q = ws_inputs.normal_bf16((N, d), 3.0, 3, 0, DEV)
    K = ws_inputs.normal_bf16((M, d), 3.0, 3, 1, DEV)
    V = ws_inputs.normal_bf16((M, d), 1.0, 3, 2, DEV)
    O = lib.recurrence_attention(Q, K, V)
    check(O, attn.attention(f64(Q), f64(K), f64(V)), f64(V))


def test_closed_forms(lib):
    d = 64
    # (The weight of the top key is exp2(fma(s, c, -round(s*c))), which is 1 only to within 2^-23 or so:
    # the closed forms below hold to fp32 rounding, not bit for bit.)
    # one key: O = V_0
    Q = ws_inputs.normal_bf16((130, d), 1.0, 4, 0, DEV)
    K = ws_inputs.normal_bf16((1, d), 1.0, 4, 1, DEV)
    V = ws_inputs.normal_bf16((1, d), 1.0, 4, 2, DEV)
    O = lib.recurrence_attention(Q, K, V)
    assert torch.allclose(O, V.float().expand(130, d), rtol=2e-6, atol=0)
    # Q = 0: all scores are exactly 0, all weights exactly 1, the sum exactly M: O is the mean of the rows of V
    M = 200
    Q = torch.zeros((70, d), dtype=torch.bfloat16, device=DEV)
    K = ws_inputs.normal_bf16((M, d), 1.0, 5, 1, DEV)
    V = ws_inputs.small_int_bf16((M, d), 8, 5, 2, DEV)          # integer V: the sums are exact in fp32
    O = lib.recurrence_attention(Q, K, V)
    mean = (V.double().sum(dim=0) / M).float()
    assert torch.equal(O, mean.expand(70, d))
    # a dominant key takes all the weight
    d = 128
    Q = torch.zeros((64, d), dtype=torch.bfloat16, device=DEV); Q[:, 0] = 48.0
    K = torch.zeros((300, d), dtype=torch.bfloat16, device=DEV); K[211, 0] = 48.0; K[5, 0] = 40.0
    V = ws_inputs.normal_bf16((300, d), 1.0, 6, 2, DEV)
    O = lib.recurrence_attention(Q, K, V)
    # the runner-up's weight is exp(-34); the top weight is 1 to within 2^-24 * |score * log2 e| = 2e-5 here
    assert torch.allclose(O, V[211].float().expand(64, d), rtol=1e-4, atol=1e-6)


def test_two_calls_give_identical_bits_and_batches_are_independent(lib):
    batch, N, M, d = 4, 200, 333, 128
    Q = ws_inputs.normal_bf16((batch, N, d), 1.0, 7, 0, DEV)
    K = ws_inputs.normal_bf16((batch, M, d), 1.0, 7, 1, DEV)
    V = ws_inputs.normal_bf16((batch, M, d), 1.0, 7, 2, DEV)
    O1 = lib.recurrence_attention(Q, K, V)
    O2 = lib.recurrence_attention(Q, K, V)
    assert torch.equal(O1, O2)
    for b in range(batch):
        assert torch.equal(lib.recurrence_attention(Q[b].contiguous(), K[b].contiguous(), V[b].contiguous()), O1[b])


def test_output_is_not_written_outside_its_rows(lib):
    N, M, d = 70, 100, 64
    Q = ws_inputs.normal_bf16((N, d), 1.0, 8, 0, DEV)
    K = ws_inputs.normal_bf16((M, d), 1.0, 8, 1, DEV)
    V = ws_inputs.normal_bf16((M, d), 1.0, 8, 2, DEV)
    guard = torch.full((N + 2, d), -777.0, dtype=torch.float32, device=DEV)
    lib.recurrence_attention(Q, K, V, out=guard[1:N + 1])
    assert bool((guard[0] == -777.0).all()) and bool((guard[N + 1] == -777.0).all())
    assert bool((guard[1:N + 1] != -777.0).all())


def test_errors(lib):
    Q = torch.zeros((4, 32), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(lib.CycError):
        lib.recurrence_attention(Q, Q, Q)                       # d = 32 is not supported
    f = lib.cyc_recurrence_attention
    assert f(0x1000, 0x2000, 0x3000, 0x4000, 1, 4, 0, 64) == 2  # no keys
    assert f(0x1000, 0x2000, 0x3000, 0x1000, 1, 4, 4, 64) == 4  # O aliases Q
    assert f(0, 0, 0, 0, 0, 4, 4, 64) == 0                      # empty batch


def test_full_size_sampled_queries(lib, attn):
    """The benchmark's configuration (batch 64, N = M = 4096, d = 128); queries are independent of one
    another, so the oracle checks a sample of them in a few batch elements."""
    w = ws_inputs.ATTN_WORKLOADS["f1_attn_4096"]
    assert (w.batch, w.N, w.M, w.d) == (64, 4096, 4096, 128)
    Q, K, V = ws_inputs.make_attn_inputs(w, DEV)
    O = lib.recurrence_attention(Q, K, V)
    torch.cuda.synchronize()
    rows = [0, 1, 63, 64, 255, 256, 1000, 2047, 4032, 4095]
    for b in (0, 17, 63):
        ref = attn.attention(f64(Q[b][rows]), f64(K[b]), f64(V[b]))
        check(O[b][rows], ref, f64(V[b]))
    # every row is a weighted mean of V: inside the hull of V in every coordinate
    assert bool((O <= V.float().amax(dim=1, keepdim=True) + 1e-2).all())
    assert bool((O >= V.float().amin(dim=1, keepdim=True) - 1e-2).all())


def test_full_size_head_dimension_64(lib, attn):
    """The other kernel instantiation (d = 64, 128-key tiles) at the benchmark's batch and sequence lengths."""
    batch, N, M, d = 64, 4096, 4096, 64
    Q = ws_inputs.normal_bf16((batch, N, d), 1.0, 19, 0, DEV)
    K = ws_inputs.normal_bf16((batch, M, d), 1.0, 19, 1, DEV)
    V = ws_inputs.normal_bf16((batch, M, d), 1.0, 19, 2, DEV)
    O = lib.recurrence_attention(Q, K, V)
    torch.cuda.synchronize()
    rows = [0, 31, 32, 255, 256, 1234, 4095]
    for b in (0, 40, 63):
        ref = attn.attention(f64(Q[b][rows]), f64(K[b]), f64(V[b]))
        check(O[b][rows], ref, f64(V[b]))
    assert bool((O <= V.float().amax(dim=1, keepdim=True) + 1e-2).all())
    assert bool((O >= V.float().amin(dim=1, keepdim=True) - 1e-2).all())
