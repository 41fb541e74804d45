"""ctypes binding of libcyclotron_mm.so.  Same names as the C ABI (include/cyclotron_mm.h).

PyTorch appears here only as the owner of device memory and streams.  There is no
fallback: if the shared library is missing, the first call raises ImportError.
"""
from __future__ import annotations

import ctypes
import os

CYC_BF16_F32 = 0
CYC_I8_I32 = 1
CYC_OK = 0

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libcyclotron_mm.so")


def lib_path() -> str:
    return _LIB_PATH


def _load() -> ctypes.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is not built; run `python -m paper_2511_09987_amd.build` "
                          "(needs hipcc, cross-compiles for gfx950)")
    lib = ctypes.CDLL(_LIB_PATH)
    i64, ptr, cint = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    lib.cyc_recurrence_matmul.argtypes = [ptr, ptr, ptr, i64, i64, i64, cint, ptr]
    lib.cyc_recurrence_matmul.restype = cint
    lib.cyc_recurrence_matmul_noalloc.argtypes = [ptr, ptr, ptr, i64, i64, i64, cint, ptr]
    lib.cyc_recurrence_matmul_noalloc.restype = cint
    lib.cyc_recurrence_matmul_batched.argtypes = [ptr, ptr, ptr, i64, i64, i64, i64, i64, i64, i64, cint, ptr]
    lib.cyc_recurrence_matmul_batched.restype = cint
    lib.cyc_recurrence_trsm.argtypes = [ptr, ptr, ptr, ptr, i64, i64, i64, ptr]
    lib.cyc_recurrence_trsm.restype = cint
    lib.cyc_recurrence_cholesky.argtypes = [ptr, ptr, ptr, i64, i64, ptr]
    lib.cyc_recurrence_cholesky.restype = cint
    lib.cyc_recurrence_attention.argtypes = [ptr, ptr, ptr, ptr, i64, i64, i64, i64, ptr]
    lib.cyc_recurrence_attention.restype = cint
    lib.cyc_status_string.argtypes = [cint]
    lib.cyc_status_string.restype = ctypes.c_char_p
    lib.cyc_version.argtypes = []
    lib.cyc_version.restype = cint
    lib.cyc_kernel_name.argtypes = [ptr, ptr, ptr, i64, i64, i64, i64, i64, i64, i64, cint]
    lib.cyc_kernel_name.restype = ctypes.c_char_p
    lib.cyc_force_kernel.argtypes = [ctypes.c_char_p]
    lib.cyc_force_kernel.restype = cint
    lib.cyc_diag_mfma_ceiling.argtypes = [cint, cint, i64, ptr, ctypes.POINTER(ctypes.c_double), ptr]
    lib.cyc_diag_mfma_ceiling.restype = cint
    lib.cyc_diag_issue_mix.argtypes = [cint, cint, cint, cint, i64, ptr, ctypes.POINTER(ctypes.c_double), ptr]
    lib.cyc_diag_issue_mix.restype = cint
    lib.cyc_diag_mfma_f32_tiles.argtypes = [ptr, ptr, ptr, ptr, i64, ptr]
    lib.cyc_diag_mfma_f32_tiles.restype = cint
    lib.cyc_diag_set_wait_limit.argtypes = [i64]
    lib.cyc_diag_set_wait_limit.restype = cint
    lib.cyc_diag_clock.argtypes = [ptr, i64, ptr]
    lib.cyc_diag_clock.restype = cint
    return lib


_cached = None


def _lib() -> ctypes.CDLL:
    """The loaded library; loading is deferred to first use so that the build module can be
    imported before the library exists.  Raises ImportError if it is not built."""
    global _cached
    if _cached is None:
        _cached = _load()
    return _cached


class CycError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(cyc_status_string(status))


def cyc_status_string(status: int) -> str:
    return _lib().cyc_status_string(int(status)).decode()


def cyc_version() -> int:
    return int(_lib().cyc_version())


def cyc_recurrence_matmul(A: int, B: int, C: int, M: int, K: int, N: int, dtype: int, stream: int = 0) -> int:
    """Raw call: device addresses as ints, returns the cyc_status."""
    return int(_lib().cyc_recurrence_matmul(A, B, C, M, K, N, dtype, stream))


def cyc_recurrence_matmul_noalloc(A: int, B: int, C: int, M: int, K: int, N: int, dtype: int, stream: int = 0) -> int:
    """Raw call of the allocation-free variant: device addresses as ints, returns the cyc_status."""
    return int(_lib().cyc_recurrence_matmul_noalloc(A, B, C, M, K, N, dtype, stream))


def cyc_recurrence_matmul_batched(A: int, B: int, C: int, batch: int, M: int, K: int, N: int,
                                  strideA: int, strideB: int, strideC: int, dtype: int, stream: int = 0) -> int:
    return int(_lib().cyc_recurrence_matmul_batched(A, B, C, batch, M, K, N, strideA, strideB, strideC,
                                                  dtype, stream))


def cyc_recurrence_trsm(L: int, B: int, X: int, Xh: int, n: int, nrhs: int, nb: int, stream: int = 0) -> int:
    """Raw call: device addresses as ints, returns the cyc_status."""
    return int(_lib().cyc_recurrence_trsm(L, B, X, Xh, n, nrhs, nb, stream))


def cyc_recurrence_attention(Q: int, K: int, V: int, O: int, batch: int, N: int, M: int, d: int, stream: int = 0) -> int:
    """Raw call: device addresses as ints, returns the cyc_status."""
    return int(_lib().cyc_recurrence_attention(Q, K, V, O, batch, N, M, d, stream))


def cyc_kernel_name(A: int, B: int, C: int, batch: int, M: int, K: int, N: int,
                    strideA: int, strideB: int, strideC: int, dtype: int) -> str:
    return _lib().cyc_kernel_name(A, B, C, batch, M, K, N, strideA, strideB, strideC, dtype).decode()


def cyc_force_kernel(name) -> int:
    """Force a kernel family by name (None or "": back to the dispatcher); returns the cyc_status."""
    return int(_lib().cyc_force_kernel((name or "").encode()))


def cyc_diag_mfma_ceiling(dtype: int, mfma_shape: int, iters: int, sink: int, stream: int = 0):
    """Raw call; returns (cyc_status, operations of the launch)."""
    ops = ctypes.c_double(0.0)
    st = int(_lib().cyc_diag_mfma_ceiling(dtype, mfma_shape, iters, sink, ctypes.byref(ops), stream))
    return st, ops.value


def cyc_diag_issue_mix(mfma_shape: int, other_kind: int, others_per_round: int, waves_per_simd: int, iters: int, sink: int,
                       stream: int = 0):
    """Raw call; returns (cyc_status, MFMA operations of the launch)."""
    ops = ctypes.c_double(0.0)
    st = int(_lib().cyc_diag_issue_mix(mfma_shape, other_kind, others_per_round, waves_per_simd, iters, sink, ctypes.byref(ops), stream))
    return st, ops.value


def cyc_diag_mfma_f32_tiles(A: int, B: int, C: int, D: int, tiles: int, stream: int = 0) -> int:
    return int(_lib().cyc_diag_mfma_f32_tiles(A, B, C, D, tiles, stream))


def cyc_diag_set_wait_limit(polls: int) -> int:
    return int(_lib().cyc_diag_set_wait_limit(polls))


def cyc_diag_clock(out: int, microseconds: int, stream: int = 0) -> int:
    return int(_lib().cyc_diag_clock(out, microseconds, stream))


def recurrence_matmul(A, B, out=None, stream=None):
    """Tensor-level convenience: C = weight-stationary recurrence of A against B.

    A: (M,K) or (batch,M,K); B: (K,N) or (batch,K,N); contiguous CUDA tensors, both
    torch.bfloat16 (C float32) or both torch.int8 (C int32).  Only allocates C and
    forwards pointers to the C ABI on the current (or given) stream.
    """
    import torch
    if not (A.is_cuda and B.is_cuda):
        raise ValueError("A and B must be device tensors; there is no CPU path")
    if A.dtype != B.dtype or A.dtype not in (torch.bfloat16, torch.int8):
        raise ValueError("A and B must both be bfloat16 or both int8")
    if A.dim() != B.dim() or A.dim() not in (2, 3) or not (A.is_contiguous() and B.is_contiguous()):
        raise ValueError("A and B must be contiguous and both 2-D or both 3-D")
    dtype = CYC_BF16_F32 if A.dtype == torch.bfloat16 else CYC_I8_I32
    batch = A.shape[0] if A.dim() == 3 else 1
    M, K = A.shape[-2:]
    K2, N = B.shape[-2:]
    if K != K2 or (A.dim() == 3 and B.shape[0] != batch):
        raise ValueError(f"shape mismatch: A {tuple(A.shape)}, B {tuple(B.shape)}")
    cshape = (batch, M, N) if A.dim() == 3 else (M, N)
    cdtype = torch.float32 if dtype == CYC_BF16_F32 else torch.int32
    if out is None:
        out = torch.empty(cshape, dtype=cdtype, device=A.device)
    elif tuple(out.shape) != cshape or out.dtype != cdtype or not out.is_contiguous() or out.device != A.device:
        raise ValueError("out has the wrong shape, dtype, layout or device")
    s = (stream if stream is not None else torch.cuda.current_stream(A.device)).cuda_stream
    st = cyc_recurrence_matmul_batched(A.data_ptr(), B.data_ptr(), out.data_ptr(), batch, M, K, N,
                                       M * K, K * N, M * N, dtype, s)
    if st != CYC_OK:
        raise CycError(st)
    return out


def cyc_recurrence_cholesky(A: int, L: int, Lh: int, n: int, nb: int, stream: int = 0) -> int:
    """Raw C-ABI call: device pointers as integers, returns the status code."""
    return int(_lib().cyc_recurrence_cholesky(A, L, Lh, n, nb, stream))


def recurrence_cholesky(A, nb: int = 64, out=None, out_bf16=None, stream=None):
    """Tensor-level convenience: (L, Lh) with A = L L^T factored tile by tile (tiles of nb).

    A: (n,n) torch.float32 contiguous CUDA tensor, symmetric positive definite (its lower triangle is what counts).
    Allocates L (fp32, zero above the diagonal) and Lh (bf16, both triangles filled) unless given and forwards
    pointers to the C ABI on the current (or given) stream.
    """
    import torch
    if not A.is_cuda:
        raise ValueError("A must be a device tensor; there is no CPU path")
    if A.dtype != torch.float32 or A.dim() != 2 or A.shape[0] != A.shape[1] or not A.is_contiguous():
        raise ValueError(f"A must be a contiguous square float32 matrix, got {tuple(A.shape)} {A.dtype}")
    n = A.shape[0]
    if out is None:
        out = torch.empty((n, n), dtype=torch.float32, device=A.device)
    if out_bf16 is None:
        out_bf16 = torch.empty((n, n), dtype=torch.bfloat16, device=A.device)
    for t, dt in ((out, torch.float32), (out_bf16, torch.bfloat16)):
        if tuple(t.shape) != (n, n) or t.dtype != dt or not t.is_contiguous() or t.device != A.device:
            raise ValueError("out / out_bf16 has the wrong shape, dtype, layout or device")
    s = (stream if stream is not None else torch.cuda.current_stream(A.device)).cuda_stream
    st = cyc_recurrence_cholesky(A.data_ptr(), out.data_ptr(), out_bf16.data_ptr(), n, nb, s)
    if st != CYC_OK:
        raise CycError(st)
    return out, out_bf16


def recurrence_trsm(L, B, nb: int = 64, out=None, out_bf16=None, stream=None):
    """Tensor-level convenience: (X, Xh) with L X = B solved tile by tile (tiles of nb rows).

    L: (n,n) torch.bfloat16, B: (n,nrhs) torch.float32, contiguous CUDA tensors.  Allocates X (fp32)
    and Xh (bf16) unless given and forwards pointers to the C ABI on the current (or given) stream.
    """
    import torch
    if not (L.is_cuda and B.is_cuda):
        raise ValueError("L and B must be device tensors; there is no CPU path")
    if L.dtype != torch.bfloat16 or B.dtype != torch.float32:
        raise ValueError("L must be bfloat16 and B float32")
    if L.dim() != 2 or B.dim() != 2 or L.shape[0] != L.shape[1] or B.shape[0] != L.shape[0]:
        raise ValueError(f"shape mismatch: L {tuple(L.shape)}, B {tuple(B.shape)}")
    if not (L.is_contiguous() and B.is_contiguous()):
        raise ValueError("L and B must be contiguous")
    n, nrhs = B.shape
    if out is None:
        out = torch.empty((n, nrhs), dtype=torch.float32, device=L.device)
    if out_bf16 is None:
        out_bf16 = torch.empty((n, nrhs), dtype=torch.bfloat16, device=L.device)
    for t, dt in ((out, torch.float32), (out_bf16, torch.bfloat16)):
        if tuple(t.shape) != (n, nrhs) or t.dtype != dt or not t.is_contiguous() or t.device != L.device:
            raise ValueError("out / out_bf16 has the wrong shape, dtype, layout or device")
    s = (stream if stream is not None else torch.cuda.current_stream(L.device)).cuda_stream
    st = cyc_recurrence_trsm(L.data_ptr(), B.data_ptr(), out.data_ptr(), out_bf16.data_ptr(), n, nrhs, nb, s)
    if st != CYC_OK:
        raise CycError(st)
    return out, out_bf16


def recurrence_attention(Q, K, V, out=None, stream=None):
    """Tensor-level convenience: O = softmax(Q K^T / sqrt(d)) V by the tile recurrence.

    Q: (N,d) or (batch,N,d); K, V: (M,d) or (batch,M,d); contiguous torch.bfloat16 CUDA tensors, d 64 or 128.
    Allocates O (float32) unless given and forwards pointers to the C ABI on the current (or given) stream.
    """
    import torch
    if not (Q.is_cuda and K.is_cuda and V.is_cuda):
        raise ValueError("Q, K and V must be device tensors; there is no CPU path")
    if not (Q.dtype == K.dtype == V.dtype == torch.bfloat16):
        raise ValueError("Q, K and V must be bfloat16")
    if Q.dim() not in (2, 3) or K.dim() != Q.dim() or K.shape != V.shape or Q.shape[-1] != K.shape[-1]:
        raise ValueError(f"shape mismatch: Q {tuple(Q.shape)}, K {tuple(K.shape)}, V {tuple(V.shape)}")
    if Q.dim() == 3 and Q.shape[0] != K.shape[0]:
        raise ValueError("batch extents differ")
    if not (Q.is_contiguous() and K.is_contiguous() and V.is_contiguous()):
        raise ValueError("Q, K and V must be contiguous")
    batch = Q.shape[0] if Q.dim() == 3 else 1
    N, d = Q.shape[-2:]
    M = K.shape[-2]
    if out is None:
        out = torch.empty(tuple(Q.shape), dtype=torch.float32, device=Q.device)
    elif tuple(out.shape) != tuple(Q.shape) or out.dtype != torch.float32 or not out.is_contiguous() or out.device != Q.device:
        raise ValueError("out has the wrong shape, dtype, layout or device")
    s = (stream if stream is not None else torch.cuda.current_stream(Q.device)).cuda_stream
    st = cyc_recurrence_attention(Q.data_ptr(), K.data_ptr(), V.data_ptr(), out.data_ptr(), batch, N, M, d, s)
    if st != CYC_OK:
        raise CycError(st)
    return out
