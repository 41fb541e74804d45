"""MI355X (gfx950) weight-stationary recurrence matmul: Python binding of libcyclotron_mm.

The binding only marshals arguments; every step of the path runs in the HIP kernels
behind the C ABI declared in include/cyclotron_mm.h.
"""
from .binding import (CYC_BF16_F32, CYC_I8_I32, CycError, cyc_diag_clock, cyc_diag_issue_mix, cyc_diag_mfma_ceiling, cyc_diag_mfma_f32_tiles, cyc_diag_set_wait_limit, cyc_force_kernel,
                      cyc_kernel_name, cyc_recurrence_attention, cyc_recurrence_cholesky, cyc_recurrence_matmul,
                      cyc_recurrence_matmul_batched, cyc_recurrence_matmul_noalloc, cyc_recurrence_trsm, cyc_status_string, cyc_version, lib_path,
                      recurrence_attention, recurrence_cholesky, recurrence_matmul, recurrence_trsm)

__all__ = ["CYC_BF16_F32", "CYC_I8_I32", "CycError", "cyc_diag_clock", "cyc_diag_issue_mix", "cyc_diag_mfma_ceiling", "cyc_diag_mfma_f32_tiles", "cyc_diag_set_wait_limit", "cyc_force_kernel",
           "cyc_kernel_name", "cyc_recurrence_attention", "cyc_recurrence_cholesky", "cyc_recurrence_matmul",
           "cyc_recurrence_matmul_batched", "cyc_recurrence_matmul_noalloc", "cyc_recurrence_trsm", "cyc_status_string", "cyc_version", "lib_path",
           "recurrence_attention", "recurrence_cholesky", "recurrence_matmul", "recurrence_trsm"]
