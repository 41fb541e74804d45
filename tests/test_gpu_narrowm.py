"""GPU parity of the narrow-M kernel ((j,k) in space: B streamed once, the few rows of A pass over it) against
the row-chain oracle, element by element, through the C ABI.

int8 is bit-exact; bf16 is within the benchmark's bound and the tighter K * 2^-23, and bit-exact on small-integer
data (every summation order gives the same fp32 bits).  Shapes cover M in {1, 7, 15, 16, 17, 31, 32}, ragged K and N
(rows stay 16-byte aligned), both forms of the kernel (adjacent column blocks per wave; k-slices joined in order),
batches, and the full size of the bench workload.
"""
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
    return pkg


def gen(mode, shape_a, shape_b, seed, kind):
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
        assert err <= Ah.shape[-1] * 2.0 ** -23, f"relative error {err:.3e} is suspicious for K={Ah.shape[-1]}"


def kernel_of(lib, mode, A, B, batch, M, K, N):
    return lib.cyc_kernel_name(A.data_ptr(), B.data_ptr(), 0x10000000000, batch, M, K, N, M * K, K * N, M * N,
                               lib.CYC_I8_I32 if mode == "i8" else lib.CYC_BF16_F32)


# (batch, M, K, N): the k-sliced form (few column blocks) ...
SLICED = [(1, 16, 8192, 8192), (1, 1, 4096, 4096), (1, 7, 2048, 1024), (1, 15, 8192, 640), (2, 16, 1056, 2064),
          (1, 17, 4096, 2048), (1, 31, 1024, 4104), (3, 32, 512, 1536), (1, 16, 64, 128), (1, 5, 16, 16),
          (1, 16, 100000, 128)]
# ... and the form with adjacent column blocks per wave (batch x ceil(N / 1024) >= 128)
WIDE = [(16, 16, 512, 8192), (128, 7, 256, 1024), (64, 32, 264, 2000), (130, 15, 128, 912), (16, 1, 1024, 8184)]


@pytest.mark.parametrize("mode", ("i8", "bf16"))
@pytest.mark.parametrize("shapes", (SLICED, WIDE), ids=("k_sliced", "column_blocks"))
def test_narrowm_kernel(lib, oracle, mode, shapes):
    with forced(lib, "narrowm"):
        for n, (batch, M, K, N) in enumerate(shapes):
            if mode == "i8":
                K, N = (K + 15) // 16 * 16, (N + 15) // 16 * 16      # int8 rows must stay 16-byte aligned
            for kind in ("default", "small"):
                A, B, Ah, Bh = gen(mode, (batch, M, K), (batch, K, N), seed=3000 + n, kind=kind)
                assert kernel_of(lib, mode, A, B, batch, M, K, N) == "narrowm", (batch, M, K, N)
                C = lib.recurrence_matmul(A, B)
                torch.cuda.synchronize()
                for b in range(batch if batch <= 3 else 2):
                    bb = b if batch <= 3 else (0, batch - 1)[b]
                    Cref = oracle.ws_rowchain(Ah[bb], Bh[bb], mode)
                    check(mode, C[bb], Cref, Ah[bb], Bh[bb], exact=(kind == "small"))


def test_narrowm_dispatch(lib):
    """The dispatcher takes this kernel by itself when B is large and A has at most 32 rows."""
    name = lambda M, K, N, batch=1: lib.cyc_kernel_name(0x100000, 0x20000000, 0x4000000000, batch, M, K, N, M * K, K * N,
                                                        M * N, lib.CYC_BF16_F32)
    assert name(16, 8192, 8192) == "narrowm"
    assert name(16, 8192, 8192, batch=32) == "narrowm"
    assert name(32, 2048, 2048) == "narrowm"
    assert name(33, 2048, 2048) != "narrowm"
    assert name(16, 128, 128) != "narrowm"                  # B too small to be worth it
    assert name(8192, 8192, 16, batch=32) == "narrow"       # the mirror-image regime keeps its own kernel


@pytest.mark.parametrize("mode", ("i8", "bf16"))
def test_narrowm_one_hot_probes(lib, mode):
    """A = a e_p e_q^T, B = b e_q e_r^T  =>  C = ab e_p e_r^T with p, q, r on and around lane, fragment, copy, step,
    wave and workgroup boundaries."""
    M, K, N = 16, 2048, 2048
    tdt = torch.int8 if mode == "i8" else torch.bfloat16
    spots = [0, 1, 3, 4, 7, 8, 15, 16, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 1023, 1024, 1025, 2047]
    rng = np.random.default_rng(6)
    with forced(lib, "narrowm"):
        for trial in range(40):
            p, q, r = int(rng.integers(0, M)), int(rng.choice(spots)), int(rng.choice(spots))
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
def test_narrowm_closed_forms_and_guards(lib, mode):
    """All-ones gives K everywhere (a dropped or doubled k step shows); a ragged call writes its M x N results and
    nothing around them; two calls give the same bits."""
    tdt = torch.int8 if mode == "i8" else torch.bfloat16
    cdt = torch.int32 if mode == "i8" else torch.float32
    for M, K, N in ((16, 8192, 2048), (9, 4112, 1040), (32, 1024, 8192)):
        A = torch.ones((M, K), dtype=tdt, device=DEV)
        B = torch.ones((K, N), dtype=tdt, device=DEV)
        guard = torch.full((M + 2, N), 777, dtype=cdt, device=DEV)
        with forced(lib, "narrowm"):
            lib.recurrence_matmul(A, B, out=guard[1:M + 1])
        assert bool((guard[1:M + 1] == K).all()), (M, K, N)
        assert bool((guard[0] == 777).all()) and bool((guard[M + 1] == 777).all())
    A, B, _, _ = gen(mode, (16, 8192), (8192, 4096), seed=31, kind="default")
    C1 = lib.recurrence_matmul(A, B)
    C2 = lib.recurrence_matmul(A, B)
    assert torch.equal(C1.view(torch.int32), C2.view(torch.int32))


def test_narrowm_workload_full_size(lib, oracle):
    """The bench workload (batch 32 x (16 x 8192)(8192 x 8192) bf16) as bench.py launches it: sampled batch elements
    and column ranges against the oracle, small-integer data bit for bit."""
    w = ws_inputs.NARROWM_WORKLOADS["m1_bf16_narrowm"]
    for kind in ("default", "small"):
        if kind == "default":
            A, B = ws_inputs.make_inputs(w, DEV)
        else:
            A = ws_inputs.small_int_bf16((w.batch, w.M, w.K), 8, 55, 0, DEV)
            B = ws_inputs.small_int_bf16((w.batch, w.K, w.N), 8, 55, 1, DEV)
        assert kernel_of(lib, "bf16", A, B, w.batch, w.M, w.K, w.N) == "narrowm"
        C = lib.recurrence_matmul(A, B)
        torch.cuda.synchronize()
        rng = np.random.default_rng(17)
        for b in (0, w.batch - 1, int(rng.integers(1, w.batch - 1))):
            for j0 in (0, w.N - 512, (int(rng.integers(1, w.N - 512)) | 1)):       # odd origin: straddles every boundary
                Ah = torch_bf16_to_bits(A[b])
                Bh = torch_bf16_to_bits(B[b][:, j0:j0 + 512].contiguous())
                Cref = oracle.ws_rowchain(Ah, Bh, "bf16")
                check("bf16", C[b][:, j0:j0 + 512], Cref, Ah, Bh, exact=(kind == "small"))
        del A, B, C
        torch.cuda.empty_cache()


def test_int8_extremes_wrap_modulo_2_32_on_every_kernel_family(lib):
    """-128 is a legal int8 value and int32 partial sums wrap: with every element -128 each C_ij is K * 2^14 mod 2^32,
    which is 0 at K = 2^18 and 16 * 2^14 at K = 2^18 + 16, whatever the kernel and its summation order."""
    cases = [("narrowm", 16, 128), ("narrowm", 9, 2048), ("mfmak", 128, 128), ("mfma128", 128, 128), ("generic", 20, 24)]
    for kernel, M, N in cases:
        for K, want in ((1 << 18, 0), ((1 << 18) + 16, 16 << 14)):
            if kernel == "mfmak" and K != 1 << 18:
                continue                               # k in space wants K a multiple of its slices
            A = torch.full((M, K), -128, dtype=torch.int8, device=DEV)
            B = torch.full((K, N), -128, dtype=torch.int8, device=DEV)
            with forced(lib, kernel):
                assert kernel_of(lib, "i8", A, B, 1, M, K, N) == kernel, (kernel, M, K, N)
                C = lib.recurrence_matmul(A, B)
            assert bool((C == want).all()), (kernel, M, K, N, int(C[0, 0]))
    # the narrow-N streaming kernel holds at most 16384 int8 values of k: 2^14 * 2^14 = 2^28 per element, no wrap yet
    A = torch.full((4096, 16384), -128, dtype=torch.int8, device=DEV)
    B = torch.full((16384, 16), -128, dtype=torch.int8, device=DEV)
    with forced(lib, "narrow"):
        assert kernel_of(lib, "i8", A, B, 1, 4096, 16384, 16) == "narrow"
        C = lib.recurrence_matmul(A, B)
    assert bool((C == 1 << 28).all())
