"""The measurement aids of the C ABI run and report what they say they do (they compute nothing that a parity test
could check: these tests only make sure that bench.py's figures rest on launches that happened)."""
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
