"""Seeded synthetic inputs for the weight-stationary recurrence matmul.

This module only draws numbers.  It holds none of the method's arithmetic (no
products, no sums over k) and is the one piece of code that both the HIP path's
callers and the CPU oracle's callers use, so that both consume byte-identical
A and B.

The generator is counter based: element `idx` of tensor `tensor_id` under `seed`
is a pure function of (seed, tensor_id, idx), computed with wrapping 64-bit
integer ops that behave the same on the CPU and on the GPU.  Tensors are filled
in chunks so that a 2^31-element operand never needs more than a few hundred MB
of temporaries.  Normal deviates go through fp32 log/cos, whose last bit may
differ between devices: a caller that needs the same values on both sides
generates once and copies (the tests do).

The five workloads are the ones the benchmark definition lists: two small
parity cases, two 8192^3 compute-bound cases and the batched narrow-stream case
in which the stationary operand A (the "weights" of the paper's Space-time
Mappings section) dwarfs the streamed B and the emitted C.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch

_MASK64 = (1 << 64) - 1


def _s64(x: int) -> int:
    """Python int -> the signed 64-bit value with the same low 64 bits."""
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


_C1 = _s64(0xBF58476D1CE4E5B9)
_C2 = _s64(0x94D049BB133111EB)
_GOLD = _s64(0x9E3779B97F4A7C15)


def _lsr(x: torch.Tensor, n: int) -> torch.Tensor:
    """Logical shift right of an int64 tensor (torch's >> is arithmetic)."""
    return (x >> n) & ((1 << (64 - n)) - 1)


def _mix64(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 finaliser on an int64 tensor, wrapping arithmetic."""
    x = (x ^ _lsr(x, 30)) * _C1
    x = (x ^ _lsr(x, 27)) * _C2
    return x ^ _lsr(x, 31)


def _mix64_py(x: int) -> int:
    x &= _MASK64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _MASK64
    return x ^ (x >> 31)


def _stream_key(seed: int, tensor_id: int) -> int:
    return _s64(_mix64_py(seed * 0x9E3779B97F4A7C15 + tensor_id + 1))


def hash_bits(seed: int, tensor_id: int, start: int, count: int, device) -> torch.Tensor:
    """64 random bits (as int64) for elements start .. start+count-1."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return _mix64(idx * _GOLD + _stream_key(seed, tensor_id))


_CHUNK = 1 << 25


def _fill(out_flat: torch.Tensor, fn, seed: int, tensor_id: int) -> None:
    n = out_flat.numel()
    for s in range(0, n, _CHUNK):
        c = min(_CHUNK, n - s)
        out_flat[s:s + c] = fn(hash_bits(seed, tensor_id, s, c, out_flat.device))


def uniform_int(shape, r: int, seed: int, tensor_id: int, device="cpu",
                dtype=torch.int8) -> torch.Tensor:
    """i.i.d. integers uniform on the closed range [-r, r]."""
    out = torch.empty(shape, dtype=dtype, device=device)
    span = 2 * r + 1

    def draw(h):
        u = _lsr(h, 32)                       # 32 uniform bits, 0 .. 2^32-1
        return ((u * span) >> 32) - r         # floor(u * span / 2^32) - r

    _fill(out.view(-1), lambda h: draw(h).to(dtype), seed, tensor_id)
    return out


def normal_bf16(shape, sigma: float, seed: int, tensor_id: int, device="cpu") -> torch.Tensor:
    """i.i.d. N(0, sigma^2) drawn in fp32 (Box-Muller), rounded to bf16 (nearest even)."""
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)

    def draw(h):
        u1 = (_lsr(h, 40) + 1).to(torch.float32) * (1.0 / (1 << 24))       # (0, 1]
        u2 = (_lsr(h, 16) & 0xFFFFFF).to(torch.float32) * (1.0 / (1 << 24))  # [0, 1)
        z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)
        return (z * sigma).to(torch.bfloat16)

    _fill(out.view(-1), draw, seed, tensor_id)
    return out


def small_int_bf16(shape, r: int, seed: int, tensor_id: int, device="cpu") -> torch.Tensor:
    """Integers uniform on [-r, r] stored as bf16 (exactly representable for r <= 256)."""
    return uniform_int(shape, r, seed, tensor_id, device, dtype=torch.int16).to(torch.bfloat16)


def normal_f32(shape, sigma: float, seed: int, tensor_id: int, device="cpu") -> torch.Tensor:
    """i.i.d. N(0, sigma^2) in fp32 (the bf16 draw before its rounding)."""
    out = torch.empty(shape, dtype=torch.float32, device=device)

    def draw(h):
        u1 = (_lsr(h, 40) + 1).to(torch.float32) * (1.0 / (1 << 24))
        u2 = (_lsr(h, 16) & 0xFFFFFF).to(torch.float32) * (1.0 / (1 << 24))
        return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2) * sigma

    _fill(out.view(-1), draw, seed, tensor_id)
    return out


def tri_lower_bf16(n: int, seed: int, tensor_id: int, device="cpu", upper=0.0) -> torch.Tensor:
    """A well-conditioned lower-triangular n x n bf16 matrix: entries below the diagonal
    N(0, (0.5/sqrt(n))^2), diagonal 1 + U[0,1); everything above the diagonal is `upper`
    (NaN there shows whether anyone reads it)."""
    L = normal_bf16((n, n), 0.5 / math.sqrt(n), seed, tensor_id, device)
    h = hash_bits(seed, tensor_id + 1000, 0, n, device)
    diag = 1.0 + _lsr(h, 40).to(torch.float32) * (1.0 / (1 << 24))
    L = torch.tril(L, -1)
    L += torch.diag(diag.to(torch.bfloat16))
    if upper != 0.0:
        L += torch.triu(torch.full((n, n), upper, dtype=torch.bfloat16, device=device), 1)
    return L


def spd_f32(n: int, seed: int, tensor_id: int, device="cpu", upper=None) -> torch.Tensor:
    """A well-conditioned symmetric positive definite n x n fp32 matrix: off-diagonal entries N(0, (0.5/sqrt(n))^2)
    mirrored across the diagonal (their spectrum stays within about [-1, 1]), diagonal 2.5 + U[0,1): eigenvalues
    in about [1.5, 4.5].  With `upper` set, everything above the diagonal is that value instead of the mirror
    image (NaN there shows whether anyone relies on it)."""
    G = torch.tril(normal_f32((n, n), 0.5 / math.sqrt(n), seed, tensor_id, device), -1)
    h = hash_bits(seed, tensor_id + 1000, 0, n, device)
    diag = 2.5 + _lsr(h, 40).to(torch.float32) * (1.0 / (1 << 24))
    A = G + torch.diag(diag)
    if upper is None:
        A += G.t()
    else:
        A += torch.triu(torch.full((n, n), upper, dtype=torch.float32, device=device), 1)
    return A


@dataclass(frozen=True)
class CholWorkload:
    """Tiled Cholesky factorisation of an n x n matrix in tiles of nb."""
    name: str
    n: int
    nb: int
    seed: int

    @property
    def ops(self) -> int:
        """n^3 / 6 multiply-adds counted as two operations each: the usual n^3 / 3."""
        return self.n ** 3 // 3


CHOL_WORKLOADS = {
    "h1_chol_8192": CholWorkload("h1_chol_8192", 8192, 64, 8),
}


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str        # "i8" (int8 -> int32) or "bf16" (bf16 -> fp32)
    batch: int
    M: int
    K: int
    N: int
    dist: str         # "uniform_int" or "normal"
    param: float      # r for uniform_int, sigma for normal
    seed: int

    @property
    def ops(self) -> int:
        """Multiply-adds counted as two operations each."""
        return 2 * self.batch * self.M * self.K * self.N

    @property
    def algorithmic_bytes(self) -> int:
        """A and B read once, C written once."""
        e_in = 1 if self.dtype == "i8" else 2
        return self.batch * ((self.M * self.K + self.K * self.N) * e_in + self.M * self.N * 4)


# sigma for the 8192^3 bf16 case: the variance is 1/sqrt(K), i.e. sigma = K^(-1/4),
# which makes Var(C_ij) = K * sigma^4 = 1.
WORKLOADS = {
    "c1_i8_64": Workload("c1_i8_64", "i8", 1, 64, 64, 64, "uniform_int", 8, 1),
    "c2_bf16_512": Workload("c2_bf16_512", "bf16", 1, 512, 512, 512, "normal", 1.0, 2),
    "c3_bf16_8192": Workload("c3_bf16_8192", "bf16", 1, 8192, 8192, 8192, "normal",
                             8192.0 ** -0.25, 3),
    "c4_i8_8192": Workload("c4_i8_8192", "i8", 1, 8192, 8192, 8192, "uniform_int", 127, 4),
    "c5_bf16_narrow": Workload("c5_bf16_narrow", "bf16", 32, 8192, 8192, 16, "normal", 1.0, 5),
}


@dataclass(frozen=True)
class TriWorkload:
    """Tiled forward solve L X = B: L n x n bf16 lower triangular, B n x nrhs fp32, tiles of nb rows."""
    name: str
    n: int
    nrhs: int
    nb: int
    seed: int

    @property
    def ops(self) -> int:
        """n(n+1)/2 multiply-adds per right-hand side, counted as two operations each."""
        return self.n * (self.n + 1) * self.nrhs

    @property
    def algorithmic_bytes(self) -> int:
        """Lower triangle of L and B read once, X (fp32) and its bf16 rounding written once."""
        return self.n * (self.n + 1) // 2 * 2 + self.n * self.nrhs * (4 + 4 + 2)


# The paper's distributed runs of the triangular solve give no sizes; the shape follows the
# compute-bound matrix-multiply workloads (8192 rows, 8192 right-hand sides).
TRI_WORKLOADS = {
    "t1_trsm_8192": TriWorkload("t1_trsm_8192", 8192, 8192, 64, 6),
}


def make_tri_inputs(w: TriWorkload, device="cpu"):
    """L (n, n) bf16 and B (n, nrhs) fp32 for a triangular-solve workload."""
    return tri_lower_bf16(w.n, w.seed, 0, device), normal_f32((w.n, w.nrhs), 1.0, w.seed, 1, device)


@dataclass(frozen=True)
class AttnWorkload:
    """Attention by the tile recurrence: `batch` independent problems, N queries, M keys, head dimension d."""
    name: str
    batch: int
    N: int
    M: int
    d: int
    seed: int

    @property
    def ops(self) -> int:
        """Two products of N x M x d multiply-adds each, counted as two operations per multiply-add."""
        return 4 * self.batch * self.N * self.M * self.d

    @property
    def algorithmic_bytes(self) -> int:
        """Q, K, V (bf16) read once, O (fp32) written once."""
        return self.batch * ((self.N + 2 * self.M) * self.d * 2 + self.N * self.d * 4)


# The paper evaluates this recurrence in simulation only and gives no sizes; batch x heads = 64,
# sequence 4096, head dimension 128 is a common shape with as many operations as the 8192^3 matmul / 2.
ATTN_WORKLOADS = {
    "f1_attn_4096": AttnWorkload("f1_attn_4096", 64, 4096, 4096, 128, 7),
}


def make_attn_inputs(w: AttnWorkload, device="cpu"):
    """Q (batch, N, d), K and V (batch, M, d), i.i.d. N(0,1) rounded to bf16 (scores then have unit variance)."""
    return (normal_bf16((w.batch, w.N, w.d), 1.0, w.seed, 0, device), normal_bf16((w.batch, w.M, w.d), 1.0, w.seed, 1, device),
            normal_bf16((w.batch, w.M, w.d), 1.0, w.seed, 2, device))


# Few output blocks and a long k extent: the shape regime of the k-in-space kernel variant.  The paper gives no
# such size; 512 x 262144 x 512 moves 0.5 GiB of operands for 1.4e11 operations (256 flop/byte: just under the
# chip's ridge of 312, so the HBM roofline bounds it).
KSPACE_WORKLOADS = {
    "k1_bf16_tallk": Workload("k1_bf16_tallk", "bf16", 1, 512, 262144, 512, "normal", 262144 ** -0.25, 9),
}


# Few rows of A over a large B: the shape regime of the (j,k)-in-space kernel variant, the mirror image of the
# narrow-stream workload (there A dominates and N = 16; here B dominates and M = 16).  batch 32 x (16 x 8192)
# (8192 x 8192): 4 GiB of B read once, 16 MiB of C.
NARROWM_WORKLOADS = {
    "m1_bf16_narrowm": Workload("m1_bf16_narrowm", "bf16", 32, 16, 8192, 8192, "normal", 1.0, 10),
}


def make_inputs(w: Workload, device="cpu", scale_down: int = 1):
    """A (batch, M, K) and B (batch, K, N) for a workload; batch dim dropped when batch == 1.

    scale_down > 1 divides M, K, N (not the narrow N) for host-sized variants of the
    same recipe.
    """
    M, K = w.M // scale_down, w.K // scale_down
    N = w.N if w.N <= 64 else w.N // scale_down
    sa = (w.batch, M, K) if w.batch > 1 else (M, K)
    sb = (w.batch, K, N) if w.batch > 1 else (K, N)
    if w.dist == "uniform_int":
        A = uniform_int(sa, int(w.param), w.seed, 0, device)
        B = uniform_int(sb, int(w.param), w.seed, 1, device)
    else:
        A = normal_bf16(sa, w.param, w.seed, 0, device)
        B = normal_bf16(sb, w.param, w.seed, 1, device)
    return A, B
