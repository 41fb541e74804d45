"""The measurement aids of the C ABI run and report what they say they do (they compute nothing that a parity test
could check: these tests only make sure that bench.py's figures rest on launches that happened)."""
import ctypes
import ctypes.util

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def lib():
    import paper_2511_09987_amd as pkg
    return pkg


def timed(fn):
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    fn()
    torch.cuda.synchronize()
    e0.record()
    fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1)


def test_mfma_ceiling_rates_are_plausible(lib):
    sink = torch.zeros(4, dtype=torch.int32, device=DEV)
    st = torch.cuda.current_stream().cuda_stream
    for dtype, peak in ((lib.CYC_BF16_F32, 2.5e15), (lib.CYC_I8_I32, 5.0e15)):
        for shape in (16, 32):
            ops = []
            ms = timed(lambda: ops.append(lib.cyc_diag_mfma_ceiling(dtype, shape, 2000, sink.data_ptr(), st)))
            assert all(o[0] == 0 for o in ops)
            rate = ops[-1][1] / (ms * 1e-3)
            assert 0.3 * peak < rate < 1.05 * peak, (dtype, shape, rate)
    assert int(sink[0]) == 0


def test_clock_probe_reads_a_plausible_clock(lib):
    out = torch.zeros(2, dtype=torch.int64, device=DEV)
    assert lib.cyc_diag_clock(out.data_ptr(), 2000, torch.cuda.current_stream().cuda_stream) == 0
    torch.cuda.synchronize()
    cycles, ticks = int(out[0]), int(out[1])
    assert ticks >= 2000 * 100
    assert 0.5 < cycles / ticks / 10 < 3.0, "engine clock in GHz"


def test_issue_mix_costs_grow_with_the_instructions_between_the_mfmas(lib):
    sink = torch.zeros(4, dtype=torch.int32, device=DEV)
    st = torch.cuda.current_stream().cuda_stream
    for shape in (16, 32):
        for waves in (1, 2):
            for kind in (0, 1, 2):
                times = []
                for per_round in (0, 32, 96):
                    ops = []
                    ms = timed(lambda: ops.append(lib.cyc_diag_issue_mix(shape, kind, per_round, waves, 1000, sink.data_ptr(), st)))
                    assert ops[-1][0] == 0 and ops[-1][1] > 0
                    times.append(ms)
                assert times[0] < times[2], (shape, waves, kind, times)         # 96 instructions per round are never free
                assert times[1] < 1.6 * times[2], (shape, waves, kind, times)
    assert int(sink[0]) == 0


def test_fp32_mfma_adds_its_four_products_like_the_scalar_chain(lib):
    """v_mfma_f32_16x16x4_f32 against d = fma(a_3, b_3, fma(a_2, b_2, fma(a_1, b_1, fma(a_0, b_0, c)))) from the C
    library's correctly rounded fmaf, bit for bit: values of ordinary size, exponents spread over 2^+-35, products and
    sums in the denormal range, and small integers with many zeros of either sign.  The Cholesky kernels rely on it."""
    libm = ctypes.CDLL(ctypes.util.find_library("m"))
    libm.fmaf.argtypes = [ctypes.c_float] * 3
    libm.fmaf.restype = ctypes.c_float
    rng = np.random.default_rng(2511)
    tiles = 24

    def floats(shape, lo, hi):
        bits = (rng.integers(0, 2, shape, dtype=np.uint32) << 31) | (rng.integers(lo, hi, shape, dtype=np.uint32) << 23) | \
            rng.integers(0, 1 << 23, shape, dtype=np.uint32)
        return bits.view(np.float32)

    cases = {
        "ordinary": (floats((tiles, 16, 4), 120, 130), floats((tiles, 4, 16), 120, 130), floats((tiles, 16, 16), 120, 132)),
        "wide exponents": (floats((tiles, 16, 4), 90, 160), floats((tiles, 4, 16), 90, 160), floats((tiles, 16, 16), 60, 190)),
        "denormal products": (floats((tiles, 16, 4), 40, 100), floats((tiles, 4, 16), 40, 100), floats((tiles, 16, 16), 1, 40)),
        "integers and signed zeros": (rng.integers(-2, 3, (tiles, 16, 4)).astype(np.float32) * np.float32(-1.0),
                                      rng.integers(-2, 3, (tiles, 4, 16)).astype(np.float32),
                                      rng.integers(-1, 2, (tiles, 16, 16)).astype(np.float32) * np.float32(-1.0)),
    }
    st = torch.cuda.current_stream().cuda_stream
    for name, (A, B, C) in cases.items():
        dA, dB, dC = (torch.from_numpy(np.ascontiguousarray(x)).to(DEV) for x in (A, B, C))
        dD = torch.empty_like(dC)
        assert lib.cyc_diag_mfma_f32_tiles(dA.data_ptr(), dB.data_ptr(), dC.data_ptr(), dD.data_ptr(), tiles, st) == 0
        D = dD.cpu().numpy()
        want = np.empty_like(C)
        for t in range(tiles):
            for i in range(16):
                for j in range(16):
                    acc = float(C[t, i, j])
                    for k in range(4):
                        acc = libm.fmaf(float(A[t, i, k]), float(B[t, k, j]), acc)
                    want[t, i, j] = acc
        same = D.view(np.uint32) == want.view(np.uint32)
        assert same.all(), f"{name}: {int((~same).sum())} of {same.size} elements differ from the ascending chain"
        if name != "integers and signed zeros":
            # the check has teeth: the same terms added in descending k give other bits somewhere
            other = np.empty_like(C)
            for t in range(2):
                for i in range(16):
                    for j in range(16):
                        acc = float(C[t, i, j])
                        for k in (3, 2, 1, 0):
                            acc = libm.fmaf(float(A[t, i, k]), float(B[t, k, j]), acc)
                        other[t, i, j] = acc
            assert (other[:2].view(np.uint32) != want[:2].view(np.uint32)).any(), name

