"""GPU parity of the tiled triangular solve (cyc_recurrence_trsm, through the C ABI) against the
CPU oracle (oracle/tri_oracle.c).

What can be compared how:
  * Integer systems (small-integer L with power-of-two diagonal, integer X, B = L X): every
    intermediate of any schedule is an exact integer, so X and Xh must match the oracle bit for bit.
  * Real data: inside a tile the library either runs the oracle's chain in the oracle's order (bit
    for bit the oracle's rows in the first tile) or, for tiles of 64 rows that its check finds well
    conditioned, multiplies by the tile's inverse in fp32, whose rows of the first tile agree with
    the oracle's within the fp32 bound of such a product, 64 * 2^-24 * (kappa^2 + kappa) max |X| with
    kappa = || |L_11^-1||L_11| ||_inf.  Later tiles go through GEMMs whose fp32 summation
    order differs from the oracle's tile-by-tile order; a last-bit difference can tip the bfloat16
    rounding of an X that later rows consume, so from the second tile on the two are compared
    against the bound both obey against the fp64 recurrence: 2 * 2^-9 * || |L^-1||L| ||_inf
    relative to max |X| (the bfloat16 rounding of X is the only error of that size).
"""
import os

import numpy as np
import pytest
import scipy.linalg
import torch

from datagen import ws_inputs
from helpers import bits_to_f64, to_bf16_bits, torch_bf16_to_bits

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def lib():
    import paper_2511_09987_amd as pkg
    assert os.path.exists(pkg.lib_path()), "libcyclotron_mm.so must be built in-tree"
    return pkg


@pytest.fixture(scope="module")
def tri():
    from oracle import tri_oracle
    return tri_oracle


def integer_system(n, nrhs, seed, density=0.2, device=DEV):
    """L (bf16), X_true (int64), B = L X_true (fp32, exact) on the device; see the pins for why
    such a system is exact in every arithmetic."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    L = torch.randint(-1, 2, (n, n), generator=g) * (torch.rand((n, n), generator=g) < density)
    L = torch.tril(L, -1)
    d = torch.tensor([1, 2, -1, 4, -2])[torch.randint(0, 5, (n,), generator=g)]
    L = L + torch.diag(d)
    X = torch.randint(-8, 9, (n, nrhs), generator=g)
    L, X = L.to(device), X.to(device)
    B = (L.double() @ X.double())
    assert float(B.abs().max()) < 2 ** 20
    return L.to(torch.bfloat16), X, B.float()


SHAPES = [(64, 64, 64), (256, 128, 64), (1000, 72, 64), (1024, 512, 128), (520, 200, 32), (1032, 264, 8),
          (37, 5, 8), (130, 33, 16), (100, 40, 10), (1, 1, 64), (1, 70, 64), (200, 1, 64), (129, 64, 128),
          # panels of 5, 7, 8 tiles, 9 = 5 + 4 and 13 = 7 + 6 tiles in the four-wave kernel (nrhs a multiple of 8, the
          # last slab partly filled); 3 and 6 tiles in the one-wave kernel (nrhs not a multiple of 8)
          (320, 72, 64), (448, 136, 64), (512, 64, 64), (576, 80, 64), (832, 200, 64), (192, 70, 64), (384, 61, 64),
          # 16 and 32 tiles: two and four full panels with the smallest products between them, a partly filled last slab
          (1024, 72, 64), (1024, 200, 64), (2048, 40, 64)]


@pytest.mark.parametrize("n,nrhs,nb", SHAPES)
def test_integer_systems_bit_exact(lib, tri, n, nrhs, nb):
    L, Xtrue, B = integer_system(n, nrhs, seed=1000 + n + nb)
    X, Xh = lib.recurrence_trsm(L, B, nb)
    torch.cuda.synchronize()
    Xo, Xho = tri.tri_tiled(torch_bf16_to_bits(L), B.cpu().numpy(), nb)
    assert np.array_equal(Xo, Xtrue.cpu().numpy().astype(np.float32)), "the oracle itself must be exact here"
    assert np.array_equal(X.cpu().numpy(), Xo), f"{int((X.cpu().numpy() != Xo).sum())} elements of X differ"
    assert np.array_equal(torch_bf16_to_bits(Xh), Xho)


def skeel(L64):
    Linv = scipy.linalg.solve_triangular(L64, np.eye(L64.shape[0]), lower=True)
    return float(np.max(np.sum(np.abs(Linv) @ np.abs(np.tril(L64)), axis=1)))


@pytest.mark.parametrize("n,nrhs,nb", [(512, 256, 64), (1024, 512, 128), (300, 100, 32), (1000, 136, 64), (77, 19, 16),
                                       (448, 72, 64), (576, 264, 64), (384, 70, 64),
                                       (1024, 264, 64), (1024, 40, 64), (2048, 72, 64)])   # full panels through the inverses with products between them
def test_real_data_against_oracle(lib, tri, n, nrhs, nb):
    L = ws_inputs.tri_lower_bf16(n, 50 + n, 0, DEV, upper=float("nan"))     # NaN above the diagonal: never read
    B = ws_inputs.normal_f32((n, nrhs), 1.0, 50 + n, 1, DEV)
    X, Xh = lib.recurrence_trsm(L, B, nb)
    torch.cuda.synchronize()
    X, Xh = X.cpu().numpy(), torch_bf16_to_bits(Xh)
    bits = torch_bf16_to_bits(L)
    Xo, Xho = tri.tri_tiled(bits, B.cpu().numpy(), nb)
    assert np.all(np.isfinite(X))
    first = min(nb, n)
    L64 = np.tril(bits_to_f64(bits))
    if not np.array_equal(X[:first], Xo[:first]):
        # only the product with the inverse may differ from the oracle's chain inside a tile, and only this much
        assert nb == 64 and n >= 64 and nrhs % 8 == 0, "this shape is solved by substitution: first tile must match bitwise"
        kappa = skeel(L64[:first, :first])
        assert np.max(np.abs(X[:first] - Xo[:first])) <= 64 * 2.0 ** -24 * (kappa * kappa + kappa) * np.max(np.abs(Xo[:first]))
    else:
        assert np.array_equal(Xh[:first], Xho[:first])
    assert np.array_equal(Xh, to_bf16_bits(X)), "Xh must be X rounded to bfloat16"
    ref = tri.tri_scalar(L64, B.cpu().numpy())
    bound = 2.0 * 2.0 ** -9 * skeel(L64) * np.max(np.abs(ref))
    assert np.max(np.abs(X - ref)) <= bound
    assert np.max(np.abs(X - Xo)) <= bound
    # the bulk agrees far better than the bound: a tipped rounding is rare
    assert np.median(np.abs(X - Xo)) <= 2.0 ** -16 * np.max(np.abs(ref))


def test_two_calls_give_identical_bits_and_inputs_are_untouched(lib):
    n, nrhs, nb = 768, 320, 64
    L = ws_inputs.tri_lower_bf16(n, 7, 0, DEV)
    B = ws_inputs.normal_f32((n, nrhs), 1.0, 7, 1, DEV)
    L0, B0 = L.clone(), B.clone()
    X1, Xh1 = lib.recurrence_trsm(L, B, nb)
    X2, Xh2 = lib.recurrence_trsm(L, B, nb)
    torch.cuda.synchronize()
    assert torch.equal(X1, X2) and torch.equal(Xh1.view(torch.int16), Xh2.view(torch.int16))
    assert torch.equal(L.view(torch.int16), L0.view(torch.int16)) and torch.equal(B, B0)


def test_tile_size_changes_where_x_is_rounded(lib, tri):
    """The hand-worked rounding case of the pins, on the GPU: nb = 1 feeds the rounded X_0 to row 1,
    nb = 2 the unrounded one."""
    L = torch.tensor([[1.0, 0.0], [1.0, 1.0]], dtype=torch.bfloat16, device=DEV)
    B = torch.tensor([[1.0 + 2.0 ** -10], [0.0]], dtype=torch.float32, device=DEV)
    X, _ = lib.recurrence_trsm(L, B, 1)
    assert X.cpu().tolist() == [[1.0 + 2.0 ** -10], [-1.0]]
    X, Xh = lib.recurrence_trsm(L, B, 2)
    assert X.cpu().tolist() == [[1.0 + 2.0 ** -10], [-(1.0 + 2.0 ** -10)]]
    assert Xh.float().cpu().tolist() == [[1.0], [-1.0]]


def test_full_size_integer_system_and_sampled_columns(lib, tri):
    """n = nrhs = 8192 in the configuration the benchmark times: an integer system checked on every
    element, and real data checked on sampled columns (columns are independent, so the oracle can
    solve just those)."""
    n = nrhs = 8192
    nb = 64
    L, Xtrue, B = integer_system(n, nrhs, seed=4242, density=0.02)
    X, Xh = lib.recurrence_trsm(L, B, nb)
    torch.cuda.synchronize()
    assert torch.equal(X, Xtrue.float()), "integer system: X differs from the exact solution"
    assert torch.equal(Xh.float(), Xtrue.float())
    cols = [0, 1, 63, 64, 4095, 8191]
    Xo, _ = tri.tri_tiled(torch_bf16_to_bits(L), B[:, cols].cpu().numpy(), nb)
    assert np.array_equal(X[:, cols].cpu().numpy(), Xo)
    del L, Xtrue, B, X, Xh

    L = ws_inputs.tri_lower_bf16(n, 99, 0, DEV)
    B = ws_inputs.normal_f32((n, nrhs), 1.0, 99, 1, DEV)
    X, Xh = lib.recurrence_trsm(L, B, nb)
    torch.cuda.synchronize()
    cols = [0, 31, 64, 1000, 4097, 8191, 5555, 77]
    Bs = B[:, cols].cpu().numpy()
    bits = torch_bf16_to_bits(L)
    Xo, Xho = tri.tri_tiled(bits, Bs, nb)
    Xs = X[:, cols].cpu().numpy()
    L64 = np.tril(bits_to_f64(bits))
    # these diagonal tiles are well conditioned (diagonal in [1, 2), off-diagonal entries of size 0.006), so the first
    # tile is a product with its inverse in fp32: within that product's bound of the oracle's chain
    kappa = skeel(L64[:nb, :nb])
    assert kappa < 2.0
    assert np.max(np.abs(Xs[:nb] - Xo[:nb])) <= 64 * 2.0 ** -24 * (kappa * kappa + kappa) * np.max(np.abs(Xo[:nb]))
    ref = tri.tri_scalar(L64, Bs)
    # || |L^-1||L| ||_inf at this size, from the solve of |L| against its own row sums (L^-1 >= 0 is not
    # given, so take the bound from the sampled columns instead): compare both to fp64 and to each other
    scale = np.max(np.abs(ref))
    err_gpu, err_orc = np.max(np.abs(Xs - ref)) / scale, np.max(np.abs(Xo - ref)) / scale
    assert err_gpu <= 4.0 * max(err_orc, 2.0 ** -9), (err_gpu, err_orc)
    assert np.max(np.abs(Xs - Xo)) / scale <= 4.0 * max(err_orc, 2.0 ** -9)
    assert np.array_equal(torch_bf16_to_bits(Xh[:, cols]), to_bf16_bits(Xs))
    # and the system is solved: residual of the fp64 check on the sampled columns
    res = np.max(np.abs(L64 @ Xs.astype(np.float64) - Bs)) / (np.max(np.abs(Bs)) + scale)
    assert res <= 2.0 ** -7, res


def test_panels_with_ill_conditioned_tiles_fall_back_to_substitution(lib, tri):
    """Tiles of 64 rows are solved through their inverses only where the library's check finds them well conditioned;
    a panel (eight tiles) that holds one ill-conditioned diagonal tile is solved by substitution as a whole.  Here
    tile 2 of a well-conditioned L gets a unit lower-triangular block of ones (its inverse has entries up to 2^62):
    the rows of the first panel, substitution all through, match the oracle bit for bit up to the first GEMM, and
    the whole solve obeys the usual bound."""
    n, nrhs, nb = 1024, 136, 64
    L = ws_inputs.tri_lower_bf16(n, 321, 0, DEV)
    bad = torch.tril(torch.ones((64, 64), dtype=torch.bfloat16, device=DEV))
    L[128:192, 128:192] = bad
    B = ws_inputs.normal_f32((n, nrhs), 1.0, 321, 1, DEV)
    X, Xh = lib.recurrence_trsm(L, B, nb)
    torch.cuda.synchronize()
    X = X.cpu().numpy()
    bits = torch_bf16_to_bits(L)
    Xo, _ = tri.tri_tiled(bits, B.cpu().numpy(), nb)
    assert np.all(np.isfinite(X))
    assert np.array_equal(X[:64], Xo[:64]), "first tile of a panel solved by substitution must match bitwise"
    L64 = np.tril(bits_to_f64(bits))
    ref = tri.tri_scalar(L64, B.cpu().numpy())
    bound = 2.0 * 2.0 ** -9 * skeel(L64) * np.max(np.abs(ref))
    assert np.max(np.abs(X - ref)) <= bound and np.max(np.abs(X - Xo)) <= bound
    assert np.array_equal(torch_bf16_to_bits(Xh), to_bf16_bits(X))


def test_zero_on_the_diagonal_gives_ieee_infinities_not_an_error(lib):
    """A zero pivot makes the tile's inverse non-finite, which the library's check rejects: the tile is solved by
    substitution and the division by zero shows as IEEE infinities or NaNs from that row on, in that tile's columns."""
    n, nrhs, nb = 512, 64, 64
    L = ws_inputs.tri_lower_bf16(n, 77, 0, DEV)
    L[70, 70] = 0.0
    B = ws_inputs.normal_f32((n, nrhs), 1.0, 77, 1, DEV)
    X, _ = lib.recurrence_trsm(L, B, nb)
    torch.cuda.synchronize()
    X = X.cpu().numpy()
    assert np.all(np.isfinite(X[:70])), "rows before the zero pivot are unaffected"
    assert not np.any(np.isfinite(X[70])), "the row of the zero pivot is a division by zero in every column"
