"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

int8 results must be bit-exact.  bf16 results must satisfy
    max_ij |C_ij - Cref_ij| / sum_k |A_ik||B_kj|  <=  2e-2
(the bound the benchmark definition states), and must be bit-exact whenever the data are
small integers, because then every partial sum is an integer below 2^24 and all summation
orders give the same fp32 value.
"""
import os

import numpy as np
import pytest
import torch

from datagen import ws_inputs
from helpers import BF16_TOL, bits_to_f64, forced, rel_err, torch_bf16_to_bits

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def lib():
    import paper_2511_09987_amd as pkg
    assert os.path.exists(pkg.lib_path()), "libcyclotron_mm.so must be built in-tree"
    return pkg


def gen(mode, shape_a, shape_b, seed, kind="default"):
    """Inputs on the GPU plus their host copies in the oracle's format."""
    if mode == "i8":
        r = 8 if kind == "small" else 127
        A = ws_inputs.uniform_int(shape_a, r, seed, 0, DEV)
        B = ws_inputs.uniform_int(shape_b, r, seed, 1, DEV)
        return A, B, A.cpu().numpy(), B.cpu().numpy()
    if kind == "small":
        A = ws_inputs.small_int_bf16(shape_a, 8, seed, 0, DEV)
        B = ws_inputs.small_int_bf16(shape_b, 8, seed, 1, DEV)
    else:
        A = ws_inputs.normal_bf16(shape_a, 1.0, seed, 0, DEV)
        B = ws_inputs.normal_bf16(shape_b, 1.0, seed, 1, DEV)
    return A, B, torch_bf16_to_bits(A), torch_bf16_to_bits(B)


def check(mode, C, Cref, Ah, Bh, exact):
    C = C.cpu().numpy()
    assert C.shape == Cref.shape and C.dtype == Cref.dtype
    if mode == "i8" or exact:
        assert np.array_equal(C, Cref), f"{int((C != Cref).sum())} of {C.size} elements differ"
    else:
        err = rel_err(C, Cref, bits_to_f64(Ah), bits_to_f64(Bh))
        assert err <= BF16_TOL, f"relative error {err:.3e} above {BF16_TOL}"
        # a correct fp32 accumulation of K terms stays below K * 2^-23 on this metric
        assert err <= Ah.shape[-1] * 2.0 ** -23, f"relative error {err:.3e} is suspicious for K={Ah.shape[-1]}"


def run_case(lib, oracle, mode, M, K, N, seed, kind="default", force=None, expect_kernel=None):
    A, B, Ah, Bh = gen(mode, (M, K), (K, N), seed, kind)
    with forced(lib, force):
        if expect_kernel:
            C0 = torch.empty((M, N), dtype=torch.int32 if mode == "i8" else torch.float32, device=DEV)
            name = lib.cyc_kernel_name(A.data_ptr(), B.data_ptr(), C0.data_ptr(), 1, M, K, N, 0, 0, 0,
                                       lib.CYC_I8_I32 if mode == "i8" else lib.CYC_BF16_F32)
            assert name == expect_kernel, f"dispatcher chose {name}, test is written for {expect_kernel}"
        C = lib.recurrence_matmul(A, B)
        torch.cuda.synchronize()
    Cref = oracle.ws_rowchain(Ah, Bh, mode)
    check(mode, C, Cref, Ah, Bh, exact=(kind == "small"))
    return C


# ---------------------------------------------------------------- config 1 and 2, in full
def test_config1_int8_64_against_literal_cell_grid(lib, oracle):
    w = ws_inputs.WORKLOADS["c1_i8_64"]
    A, B = ws_inputs.make_inputs(w, DEV)
    C = lib.recurrence_matmul(A, B)
    Cref = oracle.ws_cells(A.cpu().numpy(), B.cpu().numpy(), "i8")
    assert np.array_equal(C.cpu().numpy(), Cref)


def test_config2_bf16_512(lib, oracle):
    w = ws_inputs.WORKLOADS["c2_bf16_512"]
    A, B = ws_inputs.make_inputs(w, DEV)
    C = lib.recurrence_matmul(A, B)
    Ah, Bh = torch_bf16_to_bits(A), torch_bf16_to_bits(B)
    Cref = oracle.ws_rowchain(Ah, Bh, "bf16")
    check("bf16", C, Cref, Ah, Bh, exact=False)


# ------------------------------------------------ ragged and tiny shapes (generic kernel)
RAGGED = [(1, 1, 1), (1, 37, 1), (17, 33, 5), (5, 1, 7), (63, 64, 65), (65, 15, 63), (255, 129, 257),
          (130, 300, 70), (3, 1000, 2), (64, 64, 64), (100, 8, 100)]


@pytest.mark.parametrize("mode", ("i8", "bf16"))
def test_ragged_shapes(lib, oracle, mode):
    for n, (M, K, N) in enumerate(RAGGED):
        run_case(lib, oracle, mode, M, K, N, seed=1000 + n)
        run_case(lib, oracle, mode, M, K, N, seed=2000 + n, kind="small")


@pytest.mark.parametrize("mode", ("i8", "bf16"))
def test_generic_kernel_on_tile_multiple_shapes(lib, oracle, mode):
    run_case(lib, oracle, mode, 256, 256, 256, seed=31, force="generic", expect_kernel="generic")


# ----------------------------------------------------------------------- MFMA kernels
MFMA128 = [(128, 128, 128), (128, 256, 128), (256, 128, 384), (384, 640, 128), (512, 512, 512)]
MFMA256 = [(256, 128, 256), (256, 256, 256), (512, 384, 256), (256, 1024, 768), (768, 256, 512), (1280, 128, 1024)]


@pytest.mark.parametrize("mode", ("i8", "bf16"))
@pytest.mark.parametrize("tile,shapes", (("mfma128", MFMA128), ("mfma256", MFMA256),
                                         ("mfma128x32", MFMA128), ("mfma256x32", MFMA256)))
def test_mfma_tiles(lib, oracle, mode, tile, shapes):
    for n, (M, K, N) in enumerate(shapes):
        run_case(lib, oracle, mode, M, K, N, seed=3000 + n, force=tile, expect_kernel=tile)
        run_case(lib, oracle, mode, M, K, N, seed=4000 + n, kind="small", force=tile, expect_kernel=tile)


# shapes that are not multiples of the block or of the k-tile (rows stay 16-byte aligned)
MFMA_RAGGED = [(129, 72, 136), (255, 264, 264), (100, 72, 40), (300, 1000, 520), (64, 8, 64), (16, 16, 16),
               (1, 8, 8), (5, 24, 16), (257, 72, 8), (128, 136, 128), (130, 128, 128), (128, 128, 144),
               (513, 520, 392), (31, 4104, 33 * 8)]


@pytest.mark.parametrize("mode", ("i8", "bf16"))
@pytest.mark.parametrize("tile", ("mfma128", "mfma256", "mfma128x32", "mfma256x32"))
def test_mfma_ragged_shapes(lib, oracle, mode, tile):
    for n, (M, K, N) in enumerate(MFMA_RAGGED):
        if mode == "i8":                      # int8 rows need multiples of 16
            K, N = (K + 15) // 16 * 16 + (16 if n % 2 else 0), (N + 15) // 16 * 16
        run_case(lib, oracle, mode, M, K, N, seed=6000 + n, force=tile, expect_kernel=tile)
        run_case(lib, oracle, mode, M, K, N, seed=7000 + n, kind="small", force=tile, expect_kernel=tile)


def test_mfma_ragged_edges_are_not_overwritten(lib):
    """A ragged call must write its M x N results and nothing around them."""
    M, K, N = 200, 72, 136
    A, B, _, _ = gen("bf16", (M, K), (K, N), seed=81, kind="small")
    guard = torch.full((M + 2, N), -12345.0, dtype=torch.float32, device=DEV)
    C = guard[1:M + 1]
    for tile in ("mfma128", "mfma256", "mfma128x32", "mfma256x32"):
        with forced(lib, tile):
            lib.recurrence_matmul(A, B, out=C)
        assert torch.equal(C.double(), A.double() @ B.double())
        assert bool((guard[0] == -12345.0).all()) and bool((guard[M + 1] == -12345.0).all())


@pytest.mark.parametrize("mode", ("i8", "bf16"))
@pytest.mark.parametrize("tile", ("mfma128", "mfma256", "mfma256x32"))
def test_mfma_one_hot_probes(lib, tile, mode):
    """A = a e_p e_q^T, B = b e_q e_r^T  =>  C = ab e_p e_r^T, with p, q, r on and around
    lane, fragment, wave, k-tile and block boundaries."""
    M, K, N = 512, 512, 512
    tdt = torch.int8 if mode == "i8" else torch.bfloat16
    spots = [0, 1, 3, 4, 7, 8, 15, 16, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 300, 383, 384, 511]
    with forced(lib, tile):
        rng = np.random.default_rng(5)
        for trial in range(40):
            p, q, r = (int(rng.choice(spots)) for _ in range(3))
            A = torch.zeros((M, K), dtype=tdt, device=DEV)
            B = torch.zeros((K, N), dtype=tdt, device=DEV)
            A[p, q] = 3
            B[q, r] = -5
            B[(q + 1) % K, r] = 7          # must not contribute: A has nothing in column q+1
            C = lib.recurrence_matmul(A, B)
            nz = torch.nonzero(C).cpu().tolist()
            assert nz == [[p, r]], (p, q, r, nz[:5])
            assert float(C[p, r]) == -15.0


@pytest.mark.parametrize("mode", ("i8", "bf16"))
def test_closed_forms_on_gpu(lib, mode):
    """All-ones gives K everywhere (a dropped or doubled k slice is invisible to the bf16
    tolerance but not to this); identity weights pass B through unchanged."""
    tdt = torch.int8 if mode == "i8" else torch.bfloat16
    for M, K, N in ((512, 1024, 512), (256, 8192, 256), (70, 999, 33)):
        A = torch.ones((M, K), dtype=tdt, device=DEV)
        B = torch.ones((K, N), dtype=tdt, device=DEV)
        C = lib.recurrence_matmul(A, B)
        assert bool((C == K).all()), (M, K, N)
    for K, N in ((512, 256), (1024, 1024), (77, 19)):
        A = torch.eye(K, dtype=torch.float32, device=DEV).to(tdt)
        _, B, _, _ = gen(mode, (K, K), (K, N), seed=77)
        C = lib.recurrence_matmul(A, B)
        assert torch.equal(C.double(), B.double()), (K, N)


# ------------------------------------------------------------- narrow-stream kernel
NARROW = [  # (batch, M, K, N)
    (1, 64, 8192, 16), (2, 512, 8192, 16), (1, 256, 2048, 16), (1, 100, 4096, 16), (3, 33, 6144, 16),
    (1, 128, 1280, 16), (1, 48, 8, 16), (1, 64, 8192, 15), (1, 64, 4096, 1), (2, 40, 1032, 7),
    (1, 16, 8184, 16), (1, 300, 3072, 9)]


@pytest.mark.parametrize("mode", ("i8", "bf16"))
def test_narrow_kernel(lib, oracle, mode):
    with forced(lib, "narrow"):
        for n, (batch, M, K, N) in enumerate(NARROW):
            if mode == "i8":
                K = K * 2 if K % 16 else K          # int8 rows must stay 16-byte aligned
            for kind in ("default", "small"):
                A, B, Ah, Bh = gen(mode, (batch, M, K), (batch, K, N), seed=5000 + n, kind=kind)
                C0 = torch.empty((batch, M, N), dtype=torch.int32 if mode == "i8" else torch.float32, device=DEV)
                name = lib.cyc_kernel_name(A.data_ptr(), B.data_ptr(), C0.data_ptr(), batch, M, K, N, M * K, K * N,
                                           M * N, lib.CYC_I8_I32 if mode == "i8" else lib.CYC_BF16_F32)
                assert name == "narrow", (batch, M, K, N, name)
                C = lib.recurrence_matmul(A, B)
                for b in range(batch):
                    Cref = oracle.ws_rowchain(Ah[b], Bh[b], mode)
                    check(mode, C[b], Cref, Ah[b], Bh[b], exact=(kind == "small"))


@pytest.mark.parametrize("mode", ("i8", "bf16"))
def test_narrow_all_ones_and_dispatch(lib, mode):
    """The batched narrow workload picks the streaming kernel by itself; all-ones gives K."""
    tdt = torch.int8 if mode == "i8" else torch.bfloat16
    batch, M, K, N = 2, 4096, 8192, 16
    A = torch.ones((batch, M, K), dtype=tdt, device=DEV)
    B = torch.ones((batch, K, N), dtype=tdt, device=DEV)
    C = torch.empty((batch, M, N), dtype=torch.int32 if mode == "i8" else torch.float32, device=DEV)
    name = lib.cyc_kernel_name(A.data_ptr(), B.data_ptr(), C.data_ptr(), batch, M, K, N, M * K, K * N, M * N,
                               lib.CYC_I8_I32 if mode == "i8" else lib.CYC_BF16_F32)
    assert name == "narrow"
    lib.recurrence_matmul(A, B, out=C)
    assert bool((C == K).all())


# ------------------------------------------------------------ a seeded sweep of shapes
@pytest.mark.parametrize("mode", ("i8", "bf16"))
def test_seeded_sweep_of_shapes(lib, oracle, mode):
    """Forty shapes drawn from a fixed seed: extents from 1 to about 700 with every alignment class (multiples of
    16, of 8, odd), so that the dispatcher's choices and the ragged edges of every kernel are crossed in
    combinations the hand-picked lists above do not contain."""
    rng = np.random.default_rng(2511)
    for i in range(40):
        align = [1, 8, 16][int(rng.integers(0, 3))]
        M, K, N = (max(1, int(rng.integers(1, 700)) // a * a) for a in (1, align, align))
        run_case(lib, oracle, mode, M, K, N, seed=900 + i, kind="small" if i % 4 == 0 else "default")


# ------------------------------------------------------------ k in space (few output blocks, long k)
KSPACE = [(256, 8192, 256), (128, 65536, 384), (100, 4096, 80), (512, 16384, 512), (16, 32768, 16), (1024, 4096, 1024),
          (130, 12288, 272)]


@pytest.mark.parametrize("mode", ("i8", "bf16"))
def test_k_in_space_variant(lib, oracle, mode):
    """Few output blocks and a long k extent: the dispatcher maps k-slices to workgroups; their partial sums are
    added in slice order by a second kernel.  int8 stays bit-exact, bf16 within the usual bound; small-integer
    bf16 data are exact in any order of the adds."""
    for i, (M, K, N) in enumerate(KSPACE):
        run_case(lib, oracle, mode, M, K, N, seed=700 + i, expect_kernel="mfmak")
        run_case(lib, oracle, mode, M, K, N, seed=720 + i, kind="small", expect_kernel="mfmak")


def test_default_dispatch_is_bit_reproducible(lib):
    """Same inputs, same bits, on whatever kernel the dispatcher itself picks: the k-in-space shapes (whose slices
    are joined in a fixed order, no atomic adds), the tall-k bench workload, and one shape per other kernel family."""
    shapes = [(256, 8192, 256), (512, 16384, 512), (128, 65536, 384), (512, 512, 512), (1024, 1024, 1024), (16, 4096, 4096),
              (4096, 2048, 16), (100, 72, 40), (17, 33, 5)]
    for i, (M, K, N) in enumerate(shapes):
        A, B, _, _ = gen("bf16", (M, K), (K, N), seed=4100 + i)
        C1 = lib.recurrence_matmul(A, B)
        junk = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)      # what C held before must not matter
        C2 = lib.recurrence_matmul(A, B, out=junk)
        C3 = lib.recurrence_matmul(A, B)
        assert torch.equal(C1.view(torch.int32), C2.view(torch.int32)), (M, K, N)
        assert torch.equal(C1.view(torch.int32), C3.view(torch.int32)), (M, K, N)
    w = ws_inputs.KSPACE_WORKLOADS["k1_bf16_tallk"]
    A, B = ws_inputs.make_inputs(w, DEV)
    C0 = torch.empty((w.M, w.N), dtype=torch.float32, device=DEV)
    assert lib.cyc_kernel_name(A.data_ptr(), B.data_ptr(), C0.data_ptr(), 1, w.M, w.K, w.N, 0, 0, 0, lib.CYC_BF16_F32) == "mfmak"
    C1 = lib.recurrence_matmul(A, B)
    C2 = lib.recurrence_matmul(A, B)
    assert torch.equal(C1.view(torch.int32), C2.view(torch.int32))


def test_k_in_space_on_two_streams(lib):
    """Each stream has a workspace of its own: two k-in-space calls in flight on different streams do not disturb
    each other, and a later, larger problem on the same stream (which grows the workspace) is still right."""
    A1, B1, _, _ = gen("i8", (256, 8192), (8192, 256), seed=4201)
    A2, B2, _, _ = gen("i8", (384, 16384), (16384, 128), seed=4202)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    outs = []
    for rep in range(3):
        with torch.cuda.stream(s1):
            outs.append((lib.recurrence_matmul(A1, B1), A1, B1))
        with torch.cuda.stream(s2):
            outs.append((lib.recurrence_matmul(A2, B2), A2, B2))
    torch.cuda.synchronize()
    for C, A, B in outs:
        assert torch.equal(C.double(), A.double() @ B.double())
    A3, B3, _, _ = gen("i8", (512, 32768), (32768, 512), seed=4203)
    with torch.cuda.stream(s1):
        C3 = lib.recurrence_matmul(A3, B3)
    s1.synchronize()
    assert torch.equal(C3.double(), A3.double() @ B3.double())


def test_k_in_space_dispatch_limits(lib):
    name = lambda M, K, N, batch=1: lib.cyc_kernel_name(0x100000, 0x200000, 0x4000000, batch, M, K, N, M * K, K * N, M * N,
                                                        lib.CYC_BF16_F32)
    assert name(256, 8192, 256) == "mfmak"
    assert name(256, 2048, 256) != "mfmak"                # k too short
    assert name(2048, 8192, 2048) != "mfmak"              # enough output blocks to fill the chip
    assert name(256, 8192, 256, batch=4) != "mfmak"       # batched problems keep the fixed order
    with forced(lib, "mfma128"):
        assert name(256, 8192, 256) == "mfma128"             # the one-workgroup-per-block kernel stays available


def test_k_in_space_overwrites_c(lib):
    """C is an output: what it held before the call must not leak into the sums."""
    A, B, _, _ = gen("i8", (256, 8192), (8192, 256), seed=77)
    C = torch.full((256, 256), 12345, dtype=torch.int32, device=DEV)
    lib.recurrence_matmul(A, B, out=C)
    assert torch.equal(C, lib.recurrence_matmul(A, B))
    assert torch.equal(C.double(), A.double() @ B.double())


# ------------------------------------------------------------ determinism and batching
@pytest.mark.parametrize("mode", ("i8", "bf16"))
def test_run_to_run_bit_identical(lib, mode):
    for M, K, N in ((512, 512, 512), (1024, 2048, 1024), (130, 300, 70)):
        A, B, _, _ = gen(mode, (M, K), (K, N), seed=55)
        C1 = lib.recurrence_matmul(A, B)
        C2 = lib.recurrence_matmul(A, B)
        assert torch.equal(C1.view(torch.int32), C2.view(torch.int32))


@pytest.mark.parametrize("mode", ("i8", "bf16"))
def test_batched_equals_loop_of_single_calls(lib, mode):
    for batch, M, K, N in ((3, 256, 256, 256), (2, 128, 384, 128), (4, 33, 65, 17), (2, 512, 1024, 16)):
        A, B, _, _ = gen(mode, (batch, M, K), (batch, K, N), seed=66)
        C = lib.recurrence_matmul(A, B)
        for b in range(batch):
            Cb = lib.recurrence_matmul(A[b], B[b])
            assert torch.equal(C[b].view(torch.int32), Cb.view(torch.int32)), (batch, M, K, N, b)


def test_batched_shared_operands(lib):
    """strideA = 0 or strideB = 0 share one operand across the batch."""
    batch, M, K, N = 3, 128, 256, 128
    A, B, _, _ = gen("i8", (batch, M, K), (batch, K, N), seed=67)
    C = torch.empty((batch, M, N), dtype=torch.int32, device=DEV)
    s = torch.cuda.current_stream().cuda_stream
    st = lib.cyc_recurrence_matmul_batched(A.data_ptr(), B.data_ptr(), C.data_ptr(), batch, M, K, N,
                                           0, K * N, M * N, lib.CYC_I8_I32, s)
    assert st == 0
    for b in range(batch):
        assert torch.equal(C[b], lib.recurrence_matmul(A[0], B[b]))
    st = lib.cyc_recurrence_matmul_batched(A.data_ptr(), B.data_ptr(), C.data_ptr(), batch, M, K, N,
                                           M * K, 0, M * N, lib.CYC_I8_I32, s)
    assert st == 0
    for b in range(batch):
        assert torch.equal(C[b], lib.recurrence_matmul(A[b], B[0]))


# -------------------------------------------------------------- boundary behaviour
def test_degenerate_extents_and_errors(lib):
    s = torch.cuda.current_stream().cuda_stream
    A = torch.ones((4, 4), dtype=torch.int8, device=DEV)
    C = torch.full((4, 4), 9, dtype=torch.int32, device=DEV)
    f = lib.cyc_recurrence_matmul
    assert f(A.data_ptr(), A.data_ptr(), C.data_ptr(), 0, 4, 4, lib.CYC_I8_I32, s) == 0     # M == 0: no-op
    assert f(A.data_ptr(), A.data_ptr(), C.data_ptr(), 4, 4, 0, lib.CYC_I8_I32, s) == 0     # N == 0: no-op
    torch.cuda.synchronize()
    assert bool((C == 9).all())
    assert f(0, 0, C.data_ptr(), 4, 0, 4, lib.CYC_I8_I32, s) == 0                           # K == 0: zeros
    torch.cuda.synchronize()
    assert bool((C == 0).all())
    assert f(0, A.data_ptr(), C.data_ptr(), 4, 4, 4, lib.CYC_I8_I32, s) == 1                # NULL
    assert f(A.data_ptr(), A.data_ptr(), 0, 4, 4, 4, lib.CYC_I8_I32, s) == 1
    assert f(A.data_ptr(), A.data_ptr(), C.data_ptr(), -1, 4, 4, lib.CYC_I8_I32, s) == 2    # shape
    assert f(A.data_ptr(), A.data_ptr(), C.data_ptr(), 4, 4, 4, 7, s) == 3                  # dtype
    assert f(C.data_ptr(), A.data_ptr(), C.data_ptr(), 4, 4, 4, lib.CYC_I8_I32, s) == 4     # alias
    with pytest.raises(ValueError):
        lib.recurrence_matmul(A.cpu(), A.cpu())          # no CPU path
    with pytest.raises(ValueError):
        lib.recurrence_matmul(A, A.view(2, 8))           # K mismatch


def test_extents_beyond_one_launch(lib):
    """A batch longer than a grid's 65535 and more rows than 65535 blocks of 64 are legal: the call takes several
    launches.  Checked exactly against torch's integer matmul (tiny K, so the oracle's result is the plain sum)."""
    s = torch.cuda.current_stream().cuda_stream
    batch, M, K, N = 70000, 4, 4, 4
    A = ws_inputs.uniform_int((batch, M, K), 8, 301, 0, DEV)
    B = ws_inputs.uniform_int((batch, K, N), 8, 301, 1, DEV)
    C = torch.full((batch, M, N), 99, dtype=torch.int32, device=DEV)
    st = lib.cyc_recurrence_matmul_batched(A.data_ptr(), B.data_ptr(), C.data_ptr(), batch, M, K, N, M * K, K * N, M * N,
                                           lib.CYC_I8_I32, s)
    assert st == 0, lib.cyc_status_string(st)
    assert torch.equal(C, torch.bmm(A.float(), B.float()).to(torch.int32))
    M, K, N = 65535 * 64 + 70, 3, 3
    A = ws_inputs.uniform_int((M, K), 8, 302, 0, DEV)
    B = ws_inputs.uniform_int((K, N), 8, 302, 1, DEV)
    C = torch.full((M, N), 99, dtype=torch.int32, device=DEV)
    st = lib.cyc_recurrence_matmul(A.data_ptr(), B.data_ptr(), C.data_ptr(), M, K, N, lib.CYC_I8_I32, s)
    assert st == 0, lib.cyc_status_string(st)
    assert torch.equal(C, (A.float() @ B.float()).to(torch.int32))


def test_unaligned_pointers_fall_back(lib, oracle):
    """Tile-multiple shapes at odd addresses must not take the 16-byte-aligned fast path."""
    M = K = N = 256
    buf = ws_inputs.uniform_int((M * K + K * N + 8,), 127, 91, 0, DEV)
    A = buf[1:1 + M * K].view(M, K)
    B = buf[3 + M * K:3 + M * K + K * N].view(K, N)
    C = torch.empty((M, N), dtype=torch.int32, device=DEV)
    name = lib.cyc_kernel_name(A.data_ptr(), B.data_ptr(), C.data_ptr(), 1, M, K, N, 0, 0, 0, lib.CYC_I8_I32)
    assert name == "generic"
    st = lib.cyc_recurrence_matmul(A.data_ptr(), B.data_ptr(), C.data_ptr(), M, K, N, lib.CYC_I8_I32,
                                   torch.cuda.current_stream().cuda_stream)
    assert st == 0
    Cref = oracle.ws_rowchain(A.cpu().numpy(), B.cpu().numpy(), "i8")
    assert np.array_equal(C.cpu().numpy(), Cref)


def test_side_stream(lib, oracle):
    A, B, Ah, Bh = gen("i8", (256, 256), (256, 256), seed=12)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        C = lib.recurrence_matmul(A, B)
    s.synchronize()
    assert np.array_equal(C.cpu().numpy(), oracle.ws_rowchain(Ah, Bh, "i8"))
