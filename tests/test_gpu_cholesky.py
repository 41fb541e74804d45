"""GPU parity of the tiled Cholesky factorisation (cyc_recurrence_cholesky, through the C ABI) against the
CPU oracle (oracle/chol_oracle.c).

What can be compared how:
  * Integer factors (small-integer L0 with diagonal in {1, 2, 4}, A = L0 L0^T): every intermediate of any
    schedule is an exact integer, so L and Lh must equal L0 bit for bit.
  * Real data: the first panel involves no matrix product, and inside a tile column the library runs the
    oracle's chain in the oracle's order with IEEE square root and division: its columns must match bit for
    bit.  One exception: with tiles of 64 the 64 rows right below a well-conditioned diagonal tile (the tile the
    next diagonal tile waits for) are formed as the product S L_jj^-T with the tile's inverse in fp32 instead of by
    the chain; there the first panel agrees with the oracle within that product's fp32 bound,
    64 * 2^-24 * (kappa^2 + kappa) * max|L_ij| with kappa = || |L_jj^-1||L_jj| ||_inf, not bit for bit.
    Later panels go through a product whose fp32 summation order differs from the oracle's (one chain
    over all earlier tiles instead of one per tile); a last-bit difference can tip the bfloat16 rounding of an
    entry that later panels consume, so from the second panel on the two are compared against the bound both
    obey against the fp64 factor: 4 * 2^-9 * max|L| on every entry, 2^-12 * max|L| on the mean (the
    bfloat16 rounding of finished tiles is the only error of that size; the matrices are well conditioned).
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
def chol():
    from oracle import chol_oracle
    return chol_oracle


def integer_factor(n, seed):
    rng = np.random.default_rng(seed)
    L = np.tril(rng.integers(-1, 2, size=(n, n)) * (rng.random((n, n)) < 0.2), -1).astype(np.float64)
    L += np.diag(rng.choice([1.0, 2.0, 4.0], size=n))
    A = L @ L.T
    assert np.abs(A).max() < 2 ** 20
    return L, A


def run(lib, A, nb):
    L, Lh = lib.recurrence_cholesky(A, nb=nb)
    torch.cuda.synchronize()
    return L.cpu().numpy(), bits_to_f64(torch_bf16_to_bits(Lh))


def check_first_panel(L, Lh, Lo, Lho, nb):
    """Columns of the first panel against the oracle: bit for bit, except, with tiles of 64, the 64 rows below the
    diagonal tile when the library formed them through the tile's inverse (see the top of this file)."""
    n = L.shape[0]
    first = min(nb, n)
    same = np.ones(n, dtype=bool)
    if nb == 64 and n >= 128 and not np.array_equal(L[64:128, :64], Lo[64:128, :64]):
        same[64:128] = False
        L11 = Lo[:64, :64].astype(np.float64)
        inv = np.linalg.inv(L11)
        kappa = float(np.max(np.sum(np.abs(inv) @ np.abs(L11), axis=1)))
        bound = 64 * 2.0 ** -24 * (kappa * kappa + kappa) * np.abs(Lo[64:128, :64]).max()
        assert np.abs(L[64:128, :64].astype(np.float64) - Lo[64:128, :64]).max() <= bound
    assert np.array_equal(L[same][:, :first], Lo[same][:, :first]), "the first panel must match the oracle bit for bit"
    assert np.array_equal(np.tril(Lh)[same][:, :first], Lho[same][:, :first])


def check_structure(L, Lh):
    assert np.array_equal(L, np.tril(L)), "L must be zero above the diagonal"
    assert np.array_equal(Lh, Lh.T), "Lh must hold both triangles"
    assert np.all(np.abs(np.tril(Lh) - L) <= 2.0 ** -8 * np.abs(L)), "Lh must be L rounded to bfloat16"


SHAPES = [(64, 64), (128, 64), (256, 64), (1000, 64), (1024, 64), (520, 32), (264, 8), (37, 8), (130, 16), (100, 10),
          (1, 64), (63, 64), (65, 64), (200, 7), (192, 48),
          # the next diagonal tile in the rows kernel: up to a group boundary (9 tiles), two boundaries and a ragged
          # last tile (1096 = 17 x 64 + 8), and rows of Lh that are not 16-byte aligned (900: no fused path at all)
          (576, 64), (1096, 64), (900, 64),
          # three groups and more: the first diagonal tile of the third and fourth group rides along with the last panel
          # of the group before, and the group's product then writes over its place in L (restored from a copy)
          (1664, 64),
          # ... and with a single workgroup in the launch that reads the tile's copy and restores it
          (1152, 64),
          # launches whose last two workgroups take the group's earlier panels out of the next launch's first tiles: where
          # that starts and stops inside a second group (its panels 1 .. 5), next to the matrix's end (1280: the group ends
          # after five panels; 1344 and 1352: six, the second with a ragged last tile), and in a full second group
          (1280, 64), (1344, 64), (1352, 64), (2112, 64)]


@pytest.mark.parametrize("n,nb", SHAPES)
def test_integer_factors_bit_exact(lib, n, nb):
    L0, A = integer_factor(n, 100 + n + nb)
    L, Lh = run(lib, torch.from_numpy(A.astype(np.float32)).to(DEV), nb)
    assert np.array_equal(L.astype(np.float64), L0)
    assert np.array_equal(np.tril(Lh), L0)
    check_structure(L, Lh)


@pytest.mark.parametrize("n,nb", SHAPES)
def test_against_oracle(lib, chol, n, nb):
    A = ws_inputs.spd_f32(n, 200 + n, 0, DEV)
    L, Lh = run(lib, A, nb)
    An = A.cpu().numpy()
    Lo, Lho = chol.chol_tiled(An, nb)
    assert np.all(np.isfinite(L))
    check_structure(L, Lh)
    check_first_panel(L, Lh, Lo, bits_to_f64(Lho), nb)
    ref = chol.chol_scalar(An.astype(np.float64))
    scale = np.abs(ref).max()
    for name, other in (("oracle", Lo.astype(np.float64)), ("fp64", ref)):
        err = np.abs(L.astype(np.float64) - other)
        assert err.max() <= 4 * 2.0 ** -9 * scale, f"vs {name}: max error {err.max():.3e}"
        assert err.mean() <= 2.0 ** -12 * scale, f"vs {name}: mean error {err.mean():.3e}"
    if nb >= n:                                   # a single tile: nothing is rounded, nothing reordered
        assert np.array_equal(L, Lo)


def test_upper_triangle_of_a_does_not_matter(lib):
    n, nb = 300, 64
    A = ws_inputs.spd_f32(n, 7, 0, DEV)
    B = ws_inputs.spd_f32(n, 7, 0, DEV, upper=float("nan"))
    L1, H1 = run(lib, A, nb)
    L2, H2 = run(lib, B, nb)
    assert np.array_equal(L1, L2) and np.array_equal(H1, H2) and np.all(np.isfinite(L2))


def test_two_calls_give_identical_bits_and_outputs_are_fully_written(lib):
    n, nb = 520, 64
    A = ws_inputs.spd_f32(n, 8, 0, DEV)
    L1 = torch.full((n, n), float("nan"), dtype=torch.float32, device=DEV)
    H1 = torch.full((n, n), float("nan"), dtype=torch.bfloat16, device=DEV)
    lib.recurrence_cholesky(A, nb=nb, out=L1, out_bf16=H1)
    L2, H2 = lib.recurrence_cholesky(A, nb=nb)
    torch.cuda.synchronize()
    assert torch.equal(L1, L2) and torch.equal(H1.view(torch.int16), H2.view(torch.int16))
    assert bool(torch.isfinite(L1).all()) and bool(torch.isfinite(H1.float()).all())


def test_second_stream_is_ordered_with_the_callers_stream(lib):
    """Three groups of panels and more: part of the work runs on the library's second stream.  The call must still
    be ordered after what the caller's stream held before it (the fill of A) and before what follows it (the copy
    of L), on a stream that is not the default one, call after call."""
    n, nb = 1600, 64
    A0 = ws_inputs.spd_f32(n, 9, 0, DEV)
    ref_L, ref_H = lib.recurrence_cholesky(A0, nb=nb)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()          # default priority
    A = torch.zeros_like(A0)
    L = torch.empty_like(A0)
    H = torch.empty((n, n), dtype=torch.bfloat16, device=DEV)
    copies = []
    with torch.cuda.stream(side):
        for _ in range(3):
            A.zero_()
            A.copy_(A0)                                          # queued before the call
            lib.recurrence_cholesky(A, nb=nb, out=L, out_bf16=H)
            copies.append((L.clone(), H.clone()))                # queued after the call
            L.fill_(float("nan"))
    side.synchronize()
    for Lc, Hc in copies:
        assert torch.equal(Lc, ref_L) and torch.equal(Hc.view(torch.int16), ref_H.view(torch.int16))


def test_not_positive_definite_gives_nan(lib):
    A = torch.tensor([[1.0, 2.0], [2.0, 1.0]], device=DEV)
    L, Lh = run(lib, A, 1)
    assert L[0, 0] == 1.0 and L[1, 0] == 2.0 and np.isnan(L[1, 1])


def test_errors(lib):
    A = ws_inputs.spd_f32(16, 1, 0, DEV)
    with pytest.raises(lib.CycError):
        lib.recurrence_cholesky(A, nb=0)
    with pytest.raises(lib.CycError):
        lib.recurrence_cholesky(A, nb=65)
    with pytest.raises(ValueError):
        lib.recurrence_cholesky(A[:, :8].contiguous())
    L, Lh = lib.recurrence_cholesky(torch.empty((0, 0), dtype=torch.float32, device=DEV))
    assert L.shape == (0, 0)


def test_full_size_leading_block_and_reconstruction(lib, chol):
    """The benchmark's configuration (n = 8192, nb = 64).  The factor of a leading principal block is the leading
    block of the factor, so the oracle checks the first 1024 rows and columns; the whole factor must reproduce
    sampled rows of A to bfloat16 accuracy."""
    w = ws_inputs.CHOL_WORKLOADS["h1_chol_8192"]
    assert (w.n, w.nb) == (8192, 64)
    A = ws_inputs.spd_f32(w.n, w.seed, 0, DEV)
    L, Lh = lib.recurrence_cholesky(A, nb=w.nb)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(L).all())
    assert bool((torch.triu(L, 1) == 0).all())
    assert torch.equal(Lh.view(torch.int16), Lh.t().contiguous().view(torch.int16))
    k = 1024
    Lo, Lho = chol.chol_tiled(A[:k, :k].cpu().numpy(), w.nb)
    Lk = L[:k, :k].cpu().numpy()
    check_first_panel(Lk, bits_to_f64(torch_bf16_to_bits(Lh[:k, :k].contiguous())), Lo, bits_to_f64(Lho), w.nb)
    ref = chol.chol_scalar(A[:k, :k].double().cpu().numpy())
    scale = np.abs(ref).max()
    for other in (Lo.astype(np.float64), ref):
        err = np.abs(Lk.astype(np.float64) - other)
        assert err.max() <= 4 * 2.0 ** -9 * scale and err.mean() <= 2.0 ** -12 * scale
    rows = torch.tensor([0, 1, 63, 64, 1000, 4095, 4096, 8000, 8191], device=DEV)
    rec = L[rows].double() @ L.double().t()
    want = torch.tril(A.double()) + torch.tril(A.double(), -1).t()
    assert float((rec - want[rows]).abs().max()) <= 8 * 2.0 ** -9 * float(A.abs().max())


def test_rows_below_an_ill_conditioned_diagonal_tile_keep_the_chain(lib, chol):
    """The product with the inverse stands in for the chain only below a diagonal tile that passes the library's check
    (||L_jj^-1||_1 ||L_jj||_1 <= 8).  Here the first diagonal tile of the factor is the lower triangle of ones (norm
    64, inverse of norm 2): the rows below it must come from the chain, bit for bit the oracle's, and the tiles after
    it, which pass, may use the product."""
    n, nb = 512, 64
    rng = np.random.default_rng(5)
    L0 = np.tril(rng.normal(0.0, 0.5 / np.sqrt(n), size=(n, n)), -1) + np.diag(1.5 + rng.random(n))
    L0[:64, :64] = np.tril(np.ones((64, 64)))
    A = (L0 @ L0.T).astype(np.float32)
    L, Lh = run(lib, torch.from_numpy(A).to(DEV), nb)
    Lo, Lho = chol.chol_tiled(A, nb)
    assert np.all(np.isfinite(L))
    check_structure(L, Lh)
    assert np.array_equal(L[:, :64], Lo[:, :64]), "first panel, the rows below the diagonal tile included: the oracle's chain"
    ref = chol.chol_scalar(A.astype(np.float64))
    scale = np.abs(ref).max()
    err = np.abs(L.astype(np.float64) - ref)
    assert err.max() <= 4 * 2.0 ** -9 * scale * 64, "bound scaled by the norm of the ill-conditioned tile"
