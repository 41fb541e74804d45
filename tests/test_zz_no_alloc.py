"""The allocation-free entry point against the ordinary one, through the C ABI.

Both run the same kernels in the same order, so results must agree bit for bit (int8 and bf16 alike).  Two calls
in a row share the library's fixed workspace, the second with a smaller problem; a problem whose partial products do
not fit is refused with CYC_ERR_WORKSPACE and nothing enqueued.  Collected last on purpose.
"""
import numpy as np
import pytest
import torch

from datagen import ws_inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
CYC_ERR_WORKSPACE = 6


@pytest.fixture(scope="module")
def lib():
    import paper_2511_09987_amd as pkg
    return pkg


def operands(mode, M, K, N, seed):
    if mode == "i8":
        return ws_inputs.uniform_int((M, K), 127, seed, 0, DEV), ws_inputs.uniform_int((K, N), 127, seed, 1, DEV)
    return ws_inputs.normal_bf16((M, K), 1.0, seed, 0, DEV), ws_inputs.normal_bf16((K, N), 1.0, seed, 1, DEV)


@pytest.mark.parametrize("mode", ("i8", "bf16"))
def test_noalloc_matches_the_ordinary_entry_point(lib, oracle, mode):
    dt = lib.CYC_I8_I32 if mode == "i8" else lib.CYC_BF16_F32
    cdt = torch.int32 if mode == "i8" else torch.float32
    stream = torch.cuda.current_stream().cuda_stream
    # k in space (uses the fixed workspace), first a larger then a smaller problem, then shapes of the other families
    shapes = [(512, 16384, 256), (256, 8192, 128), (130, 12288, 272), (512, 512, 512), (16, 4096, 2048), (17, 33, 5)]
    for n, (M, K, N) in enumerate(shapes):
        A, B = operands(mode, M, K, N, 8800 + n)
        ref = torch.empty((M, N), dtype=cdt, device=DEV)
        assert lib.cyc_recurrence_matmul(A.data_ptr(), B.data_ptr(), ref.data_ptr(), M, K, N, dt, stream) == 0
        out = torch.full((M, N), 7, dtype=cdt, device=DEV)
        assert lib.cyc_recurrence_matmul_noalloc(A.data_ptr(), B.data_ptr(), out.data_ptr(), M, K, N, dt, stream) == 0
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int32), ref.view(torch.int32)), (mode, M, K, N)
        if n < 2 and mode == "i8":
            # and both are the oracle's result (int8: bit-exact)
            assert np.array_equal(out.cpu().numpy(), oracle.ws_rowchain(A.cpu().numpy(), B.cpu().numpy(), "i8"))
    name = lib.cyc_kernel_name(0x100000, 0x8000000, 0x40000000, 1, 512, 16384, 256, 0, 0, 0, dt)
    assert name == "mfmak", "the first two shapes are meant to run with k in space"


def test_noalloc_refuses_what_does_not_fit(lib):
    """512 x 262144 x 512 runs as 64 k-slices of 1 MiB each: twice the fixed workspace."""
    w = ws_inputs.KSPACE_WORKLOADS["k1_bf16_tallk"]
    A, B = ws_inputs.make_inputs(w, DEV)
    C = torch.full((w.M, w.N), 3.0, dtype=torch.float32, device=DEV)
    stream = torch.cuda.current_stream().cuda_stream
    st = lib.cyc_recurrence_matmul_noalloc(A.data_ptr(), B.data_ptr(), C.data_ptr(), w.M, w.K, w.N, lib.CYC_BF16_F32, stream)
    assert st == CYC_ERR_WORKSPACE, lib.cyc_status_string(st)
    torch.cuda.synchronize()
    assert bool((C == 3.0).all()), "a refused call must not touch C"
    assert "workspace" in lib.cyc_status_string(st)
