"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "cyclotron_mm.h")


@pytest.fixture(scope="module")
def pkg():
    import paper_2511_09987_amd as p
    if not os.path.exists(p.lib_path()):
        from paper_2511_09987_amd import build
        build.build()
    return p


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cyc_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_documented_entry_points():
    names = declared_functions()
    for need in ("cyc_recurrence_matmul", "cyc_recurrence_matmul_batched", "cyc_recurrence_trsm", "cyc_recurrence_attention", "cyc_recurrence_cholesky", "cyc_status_string",
                 "cyc_version"):
        assert need in names


def test_library_exports_every_declared_symbol(pkg):
    lib = ctypes.CDLL(pkg.lib_path())
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} declared in the header but not exported"


def test_status_strings_and_version(pkg):
    assert pkg.cyc_version() >= 100
    assert pkg.cyc_status_string(0) == "CYC_OK"
    for st in range(1, 7):
        assert pkg.cyc_status_string(st).startswith("CYC_ERR_")
    assert "unknown" in pkg.cyc_status_string(99)


def test_argument_validation_happens_on_the_host(pkg):
    """Every call here returns an error (or has nothing to do) before any device work."""
    f, fb = pkg.cyc_recurrence_matmul, pkg.cyc_recurrence_matmul_batched
    a, b, c = 0x10000, 0x20000, 0x30000
    assert f(a, b, c, 4, 4, 4, 9) == 3                       # unknown dtype
    assert f(a, b, c, -1, 4, 4, 0) == 2                      # negative extent
    assert f(a, b, c, 1 << 40, 1 << 40, 4, 0) == 2           # element count overflow
    assert f(0, b, c, 4, 4, 4, 0) == 1                       # NULL A
    assert f(a, b, 0, 4, 4, 4, 1) == 1                       # NULL C
    assert f(a, b, a, 4, 4, 4, 1) == 4                       # C aliases A
    assert f(a, b, b + 8, 4, 4, 4, 0) == 4                   # C overlaps B
    assert f(0, 0, 0, 0, 4, 4, 0) == 0                       # M == 0: nothing to do
    assert f(0, 0, 0, 4, 4, 0, 1) == 0                       # N == 0: nothing to do
    assert fb(a, b, c, 0, 4, 4, 4, 16, 16, 16, 0) == 0       # batch == 0
    assert fb(a, b, c, 2, 4, 4, 4, 16, 16, 8, 0) == 2        # strideC < M*N
    assert fb(a, b, c, 2, 4, 4, 4, 8, 16, 16, 0) == 2        # 0 < strideA < M*K
    assert fb(a, b, c, 2, 4, 4, 4, -16, 16, 16, 0) == 2      # negative stride


def test_dispatch_table(pkg):
    """Which kernel family serves which problem (host-only query)."""
    k = pkg.cyc_kernel_name
    A, B, C = 1 << 32, 2 << 32, 3 << 32
    assert k(A, B, C, 1, 8192, 8192, 8192, 0, 0, 0, 0) == "mfma256"
    assert k(A, B, C, 1, 8192, 8192, 8192, 0, 0, 0, 1) == "mfma256"
    assert k(A, B, C, 1, 512, 512, 512, 0, 0, 0, 0) == "mfma128"
    assert k(A, B, C, 1, 64, 64, 64, 0, 0, 0, 1) == "mfma128"
    assert k(A, B, C, 1, 8191, 8192, 8200, 0, 0, 0, 0) == "mfma256"       # ragged M and N, aligned rows
    assert k(A, B, C, 1, 100, 72, 40, 0, 0, 0, 0) == "mfma128"            # ragged everything, aligned rows
    assert k(A, B, C, 1, 1000, 1000, 1000, 0, 0, 0, 1) == "generic"       # int8 rows of 1000 bytes: not 16-byte aligned
    assert k(A, B, C, 1, 17, 33, 5, 0, 0, 0, 0) == "generic"
    assert k(A, B, C, 1, 8, 64, 4096, 0, 0, 0, 0) == "generic"            # sliver with a small B
    assert k(A, B, C, 1, 16, 8192, 8192, 0, 0, 0, 0) == "narrowm"         # few rows of A over a large B: B streamed once
    assert k(A, B, C, 32, 16, 8192, 8192, 16 * 8192, 8192 * 8192, 16 * 8192, 0) == "narrowm"
    assert k(A, B, C, 1, 7, 4096, 4096, 0, 0, 0, 1) == "narrowm"
    assert k(A, B, C, 1, 32, 4096, 4096, 0, 0, 0, 0) == "narrowm"
    assert k(A, B, C, 1, 33, 4096, 4096, 0, 0, 0, 0) != "narrowm"         # more than two 16-row blocks of A
    assert k(A, B, C, 1, 16, 8192, 8191 * 8, 0, 0, 0, 0) == "narrowm"     # ragged N, aligned rows
    assert k(A, B, C, 1, 16, 8192, 8190, 0, 0, 0, 0) != "narrowm"         # rows of B not 16-byte aligned
    assert k(A + 2, B, C, 1, 512, 512, 512, 0, 0, 0, 0) == "generic"      # unaligned A
    assert k(A, B, C, 1, 512, 0, 512, 0, 0, 0, 0) == "zero"
    assert k(A, B, C, 1, 0, 8, 512, 0, 0, 0, 0) == "none"


def test_forced_kernel_is_a_setting_of_the_library(pkg):
    """cyc_force_kernel overrides the dispatcher where the named kernel supports the problem, and gives the choice back."""
    k = pkg.cyc_kernel_name
    A, B, C = 1 << 32, 2 << 32, 3 << 32
    try:
        assert pkg.cyc_force_kernel("mfma128") == 0
        assert k(A, B, C, 1, 8192, 8192, 8192, 0, 0, 0, 0) == "mfma128"
        assert k(A, B, C, 1, 17, 33, 5, 0, 0, 0, 0) == "generic"          # mfma128 cannot serve it: the dispatcher decides
        assert pkg.cyc_force_kernel("generic") == 0
        assert k(A, B, C, 1, 8192, 8192, 8192, 0, 0, 0, 0) == "generic"
        assert pkg.cyc_force_kernel("no_such_kernel") == 2
        assert k(A, B, C, 1, 8192, 8192, 8192, 0, 0, 0, 0) == "generic"   # an unknown name changes nothing
    finally:
        assert pkg.cyc_force_kernel(None) == 0
    assert k(A, B, C, 1, 8192, 8192, 8192, 0, 0, 0, 0) == "mfma256"


def test_long_batches_and_tall_problems_are_accepted(pkg):
    """Extents beyond one launch's grid limits are legal arguments (they take several launches): no shape error
    from the planning step, which is all that runs without a device."""
    k = pkg.cyc_kernel_name
    A, B, C = 1 << 40, 2 << 40, 3 << 40
    assert k(A, B, C, 70000, 4, 4, 4, 16, 16, 16, 1) == "generic"
    assert k(A, B, C, 1, 5000000, 3, 3, 0, 0, 0, 0) == "generic"


def test_diagnostic_entry_points_validate_on_the_host(pkg):
    assert pkg.cyc_diag_mfma_ceiling(7, 16, 1000, 0x1000)[0] == 3         # unknown dtype
    assert pkg.cyc_diag_mfma_ceiling(0, 8, 1000, 0x1000)[0] == 2          # unknown MFMA shape
    assert pkg.cyc_diag_mfma_ceiling(0, 16, 1004, 0x1000)[0] == 2         # iteration count not a multiple of 8
    assert pkg.cyc_diag_mfma_ceiling(0, 16, 1000, 0)[0] == 1              # NULL sink
    assert pkg.cyc_diag_issue_mix(8, 0, 32, 1, 100, 0x1000)[0] == 2        # unknown MFMA shape
    assert pkg.cyc_diag_issue_mix(16, 3, 32, 1, 100, 0x1000)[0] == 2       # unknown instruction kind
    assert pkg.cyc_diag_issue_mix(16, 0, 24, 1, 100, 0x1000)[0] == 2       # count per round not offered
    assert pkg.cyc_diag_issue_mix(16, 0, 32, 3, 100, 0x1000)[0] == 2       # one or two waves per SIMD
    assert pkg.cyc_diag_issue_mix(16, 0, 32, 1, 0, 0x1000)[0] == 2         # no rounds
    assert pkg.cyc_diag_issue_mix(16, 0, 32, 1, 100, 0)[0] == 1            # NULL sink
    assert pkg.cyc_diag_mfma_f32_tiles(0x1000, 0x2000, 0x3000, 0x4000, -1) == 2   # negative count
    assert pkg.cyc_diag_mfma_f32_tiles(0x1000, 0x2000, 0x3000, 0, 4) == 1         # NULL result
    assert pkg.cyc_diag_mfma_f32_tiles(0x1000, 0x2002, 0x3000, 0x4000, 4) == 2    # misaligned
    assert pkg.cyc_diag_mfma_f32_tiles(0, 0, 0, 0, 0) == 0                        # nothing to do
    assert pkg.cyc_diag_set_wait_limit(-1) == 2 and pkg.cyc_diag_set_wait_limit((1 << 30) + 1) == 2
    assert pkg.cyc_diag_set_wait_limit(5) == 0 and pkg.cyc_diag_set_wait_limit(0) == 0      # set, and back to the default
    assert pkg.cyc_diag_clock(0, 100) == 1
    assert pkg.cyc_diag_clock(0x1000, 0) == 2
    assert pkg.cyc_diag_clock(0x1004, 100) == 2                           # misaligned


def test_trsm_argument_validation_happens_on_the_host(pkg):
    f = pkg.cyc_recurrence_trsm
    L, B, X, Xh = 0x100000, 0x200000, 0x300000, 0x400000
    assert f(L, B, X, Xh, -1, 4, 64) == 2                    # negative extent
    assert f(L, B, X, Xh, 8, 4, 0) == 2                      # tile size out of range
    assert f(L, B, X, Xh, 8, 4, 129) == 2
    assert f(L, B, X, Xh, 1 << 40, 1 << 40, 64) == 2         # element count overflow
    assert f(0, B, X, Xh, 8, 4, 64) == 1                     # NULL L
    assert f(L, B, X, 0, 8, 4, 64) == 1                      # NULL Xh
    assert f(L, B, B, Xh, 8, 4, 64) == 4                     # X aliases B
    assert f(L, B, X, X + 16, 8, 4, 64) == 4                 # Xh overlaps X
    assert f(L, B, L + 32, Xh, 8, 4, 64) == 4                # X overlaps L
    assert f(0, 0, 0, 0, 0, 4, 64) == 0                      # n == 0: nothing to do
    assert f(0, 0, 0, 0, 8, 0, 64) == 0                      # nrhs == 0: nothing to do


def test_cholesky_argument_validation_happens_on_the_host(pkg):
    f = pkg.cyc_recurrence_cholesky
    A, L, Lh = 0x100000, 0x200000, 0x300000
    assert f(A, L, Lh, -1, 64) == 2                          # negative extent
    assert f(A, L, Lh, 8, 0) == 2                            # tile size out of range
    assert f(A, L, Lh, 8, 65) == 2
    assert f(A, L, Lh, 1 << 40, 64) == 2                     # too large
    assert f(A + 2, L, Lh, 8, 64) == 2                       # misaligned A
    assert f(A, L, Lh + 1, 8, 64) == 2                       # misaligned Lh
    assert f(0, L, Lh, 8, 64) == 1                           # NULL A
    assert f(A, L, 0, 8, 64) == 1                            # NULL Lh
    assert f(A, A, Lh, 8, 64) == 4                           # L aliases A
    assert f(A, L, L + 64, 8, 64) == 4                       # Lh overlaps L
    assert f(A, L, A + 32, 8, 64) == 4                       # Lh overlaps A
    assert f(0, 0, 0, 0, 64) == 0                            # n == 0: nothing to do


def test_attention_argument_validation_happens_on_the_host(pkg):
    f = pkg.cyc_recurrence_attention
    Q, K, V, O = 0x100000, 0x200000, 0x300000, 0x400000
    assert f(Q, K, V, O, 1, -1, 4, 64) == 2                  # negative extent
    assert f(Q, K, V, O, 1, 4, 4, 32) == 2                   # unsupported head dimension
    assert f(Q, K, V, O, 1, 4, 0, 64) == 2                   # queries but no keys
    assert f(Q, K, V, O, 1, 1 << 40, 1 << 40, 128) == 2      # element count overflow
    assert f(Q + 2, K, V, O, 1, 4, 4, 64) == 2               # misaligned pointer
    assert f(0, K, V, O, 1, 4, 4, 64) == 1                   # NULL Q
    assert f(Q, K, V, 0, 1, 4, 4, 64) == 1                   # NULL O
    assert f(Q, K, V, K, 1, 4, 4, 64) == 4                   # O aliases K
    assert f(0, 0, 0, 0, 0, 4, 4, 64) == 0                   # empty batch: nothing to do
    assert f(0, 0, 0, 0, 2, 0, 4, 64) == 0                   # no queries: nothing to do
