"""The build checks the assembly of kernels that read LDS from inline asm: no instruction may touch the destination
registers of such a read before the wait that covers it.  Here the checker itself is checked, on small listings."""
import importlib.util
import os

HERE = os.path.dirname(os.path.abspath(__file__))
spec = importlib.util.spec_from_file_location(
    "check_async_reads", os.path.join(HERE, "..", "paper_2511_09987_amd", "check_async_reads.py"))
checker = importlib.util.module_from_spec(spec)
spec.loader.exec_module(checker)

CLEAN = """
_Zkernel:
\ts_waitcnt vmcnt(0) lgkmcnt(0)
\ts_barrier
\t;;#ASMSTART
\tds_read_b128 v[10:13], v2 offset:0x4000
\t;;#ASMEND
\tds_read_b128 v[14:17], v2 offset:0x5000
\tv_fma_f32 v20, v21, v22, v23
\ts_waitcnt lgkmcnt(1)
\tv_mfma_f32_16x16x32_bf16 v[30:33], v[10:13], v[40:43], v[30:33]
\tds_read_b128 v[10:13], v3 offset:0x4000
\ts_waitcnt lgkmcnt(1)
\tv_mfma_f32_16x16x32_bf16 v[30:33], v[14:17], v[40:43], v[30:33]
\ts_waitcnt lgkmcnt(0)
\tv_mfma_f32_16x16x32_bf16 v[30:33], v[10:13], v[40:43], v[30:33]
\ts_endpgm
"""


def test_clean_listing_passes():
    assert checker.kernels(CLEAN)[0][0] == "_Zkernel"
    assert checker.violations(CLEAN) == []


def test_copy_before_the_wait_is_found():
    bad = CLEAN.replace("\tv_fma_f32 v20, v21, v22, v23\n", "\tv_mov_b32_e32 v20, v12\n")
    found = checker.violations(bad)
    assert len(found) == 1 and "v_mov_b32_e32 v20, v12" in found[0] and "[12]" in found[0]


def test_wait_that_leaves_the_read_outstanding_is_found():
    # waiting for two outstanding operations does not cover the older of two reads
    bad = CLEAN.replace("\ts_waitcnt lgkmcnt(1)\n\tv_mfma_f32_16x16x32_bf16 v[30:33], v[10:13]",
                        "\ts_waitcnt lgkmcnt(2)\n\tv_mfma_f32_16x16x32_bf16 v[30:33], v[10:13]", 1)
    assert any("v[10:13]" in f for f in checker.violations(bad))


def test_overwrite_of_a_pending_destination_is_found():
    bad = CLEAN.replace("\tv_fma_f32 v20, v21, v22, v23\n", "\tv_fma_f32 v15, v21, v22, v23\n")
    assert len(checker.violations(bad)) == 1


def test_other_lds_operations_count_towards_the_wait():
    # a write issued after the read: "at most one outstanding" then still covers the read
    ok = CLEAN.replace("\tv_fma_f32 v20, v21, v22, v23\n", "\tds_write_b32 v5, v6\n\ts_waitcnt lgkmcnt(1)\n\tv_mov_b32_e32 v20, v12\n")
    assert checker.violations(ok) == []


def test_a_later_read_into_the_same_registers_is_allowed_but_not_its_address():
    again = CLEAN.replace("\tv_fma_f32 v20, v21, v22, v23\n", "\tds_read_b128 v[14:17], v2 offset:0x6000\n\ts_waitcnt lgkmcnt(2)\n")
    assert checker.violations(again) == []
    bad = CLEAN.replace("\tv_fma_f32 v20, v21, v22, v23\n", "\tds_read_b128 v[24:27], v15 offset:0x6000\n\ts_waitcnt lgkmcnt(2)\n")
    assert len(checker.violations(bad)) == 1
