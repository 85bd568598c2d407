"""Seeded synthetic inputs for the fused GEMM + epilogue operator.

This module only produces bytes: it holds none of the operator's arithmetic and
is the one piece that both the GPU tests/benchmark and the CPU checker are fed
from.  It depends on numpy alone, so the values do not change with the torch
version.

The paper evaluates on a public kernel benchmark whose matmul category spans
"diverse shapes" (PRAGMA, Section 4.2); that suite is not reproduced here.  The
five workloads below are dense i.i.d. stand-ins for it: small square, large
square, large low-precision square, tall-skinny with a row reduction, and a
batched tiny-output / huge-K problem.

Random numbers: a counter-based SplitMix64 stream.  Draw ``e`` of a stream with
seed ``s`` is ``mix(s + (e + 1) * 0x9E3779B97F4A7C15)``, i.e. the ``e``-th
output of the published SplitMix64 generator started at state ``s``.
  * uniform on [lo, hi): ``u = (r >> 11) * 2**-53`` then ``lo + (hi - lo) * u``
  * normal(0, std): Box-Muller on draws ``2e`` and ``2e + 1``,
    ``z = sqrt(-2 ln u1) cos(2 pi u2)`` with ``u1 = ((r1 >> 11) + 1) * 2**-53``
  * bfloat16: the float32 value rounded to nearest-even on its upper 16 bits,
    returned as uint16 bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

ACT_NONE, ACT_RELU, ACT_GELU_TANH, ACT_SILU = 0, 1, 2, 3
F32, BF16 = 0, 1

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22


def splitmix64(seed: int, start: int, count: int) -> np.ndarray:
    """Draws ``start .. start+count-1`` of the SplitMix64 stream seeded with ``seed``."""
    with np.errstate(over="ignore"):
        idx = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + idx * _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def uniform(seed: int, count: int, lo: float, hi: float) -> np.ndarray:
    """``count`` float32 values uniform on [lo, hi)."""
    out = np.empty(count, dtype=np.float32)
    for s in range(0, count, _CHUNK):
        n = min(_CHUNK, count - s)
        r = splitmix64(seed, s, n)
        u = (r >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)
        out[s:s + n] = (lo + (hi - lo) * u).astype(np.float32)
    return out


def normal(seed: int, count: int, std: float) -> np.ndarray:
    """``count`` float32 values from N(0, std**2) (std is the standard deviation)."""
    out = np.empty(count, dtype=np.float32)
    for s in range(0, count, _CHUNK):
        n = min(_CHUNK, count - s)
        r = splitmix64(seed, 2 * s, 2 * n)
        u1 = ((r[0::2] >> np.uint64(11)).astype(np.float64) + 1.0) * (2.0 ** -53)
        u2 = (r[1::2] >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)
        z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
        out[s:s + n] = (std * z).astype(np.float32)
    return out


def small_ints(seed: int, count: int, lo: int = -2, hi: int = 2) -> np.ndarray:
    """``count`` float32 values that are integers in [lo, hi] (exact in bf16 and fp32)."""
    out = np.empty(count, dtype=np.float32)
    span = np.uint64(hi - lo + 1)
    for s in range(0, count, _CHUNK):
        n = min(_CHUNK, count - s)
        r = splitmix64(seed, s, n)
        out[s:s + n] = ((r >> np.uint64(33)) % span).astype(np.float32) + np.float32(lo)
    return out


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32 exactly."""
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def fnv1a64(buf: np.ndarray) -> int:
    """FNV-1a over 64-bit words of the buffer (reproducibility checksum)."""
    b = np.ascontiguousarray(buf).view(np.uint8)
    pad = (-b.size) % 8
    if pad:
        b = np.concatenate([b, np.zeros(pad, dtype=np.uint8)])
    w = b.view(np.uint64)
    # fold words with xor/multiply in blocks so the python loop stays short
    h = np.uint64(0xCBF29CE484222325)
    prime = np.uint64(0x100000001B3)
    with np.errstate(over="ignore"):
        lanes = 4096
        padw = (-w.size) % lanes
        if padw:
            w = np.concatenate([w, np.zeros(padw, dtype=np.uint64)])
        acc = np.full(lanes, h, dtype=np.uint64)
        for row in w.reshape(-1, lanes):
            acc = (acc ^ row) * prime
        for v in acc:
            h = (h ^ v) * prime
    return int(h)


@dataclass(frozen=True)
class Dist:
    kind: str            # "uniform" | "normal" | "zero"
    a: float = 0.0       # uniform: lo ; normal: std
    b: float = 0.0       # uniform: hi


@dataclass(frozen=True)
class Workload:
    name: str
    index: int           # 1-based workload number, part of the seed
    call: str            # "fused" | "splitk"
    dtype: int           # F32 | BF16
    M: int
    N: int
    K: int
    batch: int
    A: Dist
    B: Dist
    bias: Dist
    act: int
    rowsum: bool

    @property
    def flops(self) -> float:
        return 2.0 * self.M * self.N * self.K * self.batch

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == BF16 else 4

    @property
    def algorithmic_bytes(self) -> float:
        """Read A once, read B once, read bias, write C once, write rowsum."""
        e = self.elem_bytes
        by = self.batch * (self.M * self.K + self.K * self.N + self.M * self.N) * e
        if self.bias.kind != "zero":
            by += self.N * 4
        if self.rowsum:
            by += self.batch * self.M * 4
        return float(by)


def _inv_sqrt(k: int) -> float:
    return 1.0 / float(np.sqrt(float(k)))


WORKLOADS = {
    "c1": Workload("c1", 1, "fused", F32, 256, 256, 256, 1,
                   Dist("uniform", -1.0, 1.0), Dist("uniform", -1.0, 1.0), Dist("normal", 1.0),
                   ACT_RELU, True),
    "c2": Workload("c2", 2, "fused", F32, 4096, 4096, 4096, 1,
                   Dist("uniform", -1.0, 1.0), Dist("uniform", -1.0, 1.0), Dist("normal", 0.1),
                   ACT_GELU_TANH, False),
    "c3": Workload("c3", 3, "fused", BF16, 8192, 8192, 8192, 1,
                   Dist("normal", _inv_sqrt(8192)), Dist("normal", _inv_sqrt(8192)), Dist("normal", 0.1),
                   ACT_SILU, False),
    "c4": Workload("c4", 4, "fused", BF16, 16384, 1024, 4096, 1,
                   Dist("normal", 1.0), Dist("normal", _inv_sqrt(4096)), Dist("uniform", -0.5, 0.5),
                   ACT_RELU, True),
    "c5": Workload("c5", 5, "splitk", F32, 256, 256, 65536, 16,
                   Dist("uniform", -1.0, 1.0), Dist("uniform", -1.0, 1.0), Dist("zero"),
                   ACT_NONE, True),
}

_SEED_BASE = 0x50474B0000000000  # "PGK" tag in the top bytes


def tensor_seed(workload_index: int, tensor: int, salt: int = 0) -> int:
    """Seed of tensor ``tensor`` (A=1, B=2, bias=3) of workload ``workload_index``."""
    return _SEED_BASE + 1000 * workload_index + tensor + (salt << 20)


def _draw(dist: Dist, seed: int, count: int) -> Optional[np.ndarray]:
    if dist.kind == "zero":
        return None
    if dist.kind == "uniform":
        return uniform(seed, count, dist.a, dist.b)
    if dist.kind == "normal":
        return normal(seed, count, dist.a)
    raise ValueError(dist.kind)


def make_inputs(w: Workload, salt: int = 0,
                shape: Optional[Tuple[int, int, int, int]] = None):
    """Return (A, B, bias) for workload ``w``.

    A: [batch, M, K], B: [batch, K, N]; float32, or uint16 bf16 bit patterns
    when ``w.dtype == BF16``.  bias: float32 [N] or None.  ``shape`` =
    (M, N, K, batch) overrides the sizes but keeps the distributions (used by
    reduced-size parity cases); ``salt`` selects an independent replica.
    """
    M, N, K, batch = shape if shape is not None else (w.M, w.N, w.K, w.batch)
    A = _draw(w.A, tensor_seed(w.index, 1, salt), batch * M * K)
    B = _draw(w.B, tensor_seed(w.index, 2, salt), batch * K * N)
    bias = _draw(w.bias, tensor_seed(w.index, 3, salt), N)
    if w.dtype == BF16:
        A = f32_to_bf16_bits(A)
        B = f32_to_bf16_bits(B)
    return A.reshape(batch, M, K), B.reshape(batch, K, N), bias


def make_int_inputs(dtype: int, M: int, N: int, K: int, batch: int, seed: int):
    """Integer-valued operands in {-2..2}: every summation order is exact."""
    A = small_ints(seed + 1, batch * M * K)
    B = small_ints(seed + 2, batch * K * N)
    if dtype == BF16:
        A = f32_to_bf16_bits(A)
        B = f32_to_bf16_bits(B)
    return A.reshape(batch, M, K), B.reshape(batch, K, N)


# ---- workloads of the max reduction (maximum over one dimension of a dense tensor) ----

@dataclass(frozen=True)
class ReduceWorkload:
    name: str
    index: int           # part of the seed
    dtype: int           # F32 | BF16
    shape: Tuple[int, ...]
    dim: int             # the reduced dimension

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == BF16 else 4

    @property
    def elements(self) -> int:
        n = 1
        for d in self.shape:
            n *= d
        return n

    @property
    def outputs(self) -> int:
        return self.elements // self.shape[self.dim]

    @property
    def algorithmic_bytes(self) -> float:
        """Read X once, write the values and the int32 positions once."""
        return float(self.elements * self.elem_bytes + self.outputs * (self.elem_bytes + 4))


# 1 GiB of input each: a strided reduction, the same tensor reduced along its contiguous
# dimension (short rows), a bf16 tensor, and a few very long rows.
REDUCE_WORKLOADS = {
    "r1": ReduceWorkload("r1", 11, F32, (64, 4096, 1024), 1),
    "r2": ReduceWorkload("r2", 12, F32, (64, 4096, 1024), 2),
    "r3": ReduceWorkload("r3", 13, BF16, (32, 4096, 4096), 1),
    "r4": ReduceWorkload("r4", 14, F32, (16, 1 << 24), 1),
}

_REDUCE_BLOCK = 1 << 24


def make_reduce_input(w: ReduceWorkload, salt: int = 0) -> np.ndarray:
    """Input tensor of a reduction workload: one seeded block of 2**24 values, uniform in
    [-1, 1), repeated to fill the tensor (so equal values recur 2**24 elements apart, which
    exercises the first-position rule across the whole reduced range).  float32, or uint16
    bf16 bit patterns."""
    n = w.elements
    block = uniform(tensor_seed(w.index, 1, salt), min(n, _REDUCE_BLOCK), -1.0, 1.0)
    if w.dtype == BF16:
        block = f32_to_bf16_bits(block)
    reps = (n + block.size - 1) // block.size
    return np.tile(block, reps)[:n].reshape(w.shape)


# ---- workloads of the one-dimensional convolution ----

@dataclass(frozen=True)
class ConvWorkload:
    name: str
    index: int
    dtype: int
    B: int
    Cin: int
    L: int
    Cout: int
    Kw: int
    stride: int
    pad: int
    dilation: int
    act: int

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == BF16 else 4

    @property
    def Lout(self) -> int:
        return (self.L + 2 * self.pad - self.dilation * (self.Kw - 1) - 1) // self.stride + 1

    @property
    def flops(self) -> float:
        return 2.0 * self.B * self.Cout * self.Lout * self.Cin * self.Kw

    @property
    def algorithmic_bytes(self) -> float:
        """Read x, w and bias once, write y once."""
        e = self.elem_bytes
        return float((self.B * self.Cin * self.L + self.Cout * self.Cin * self.Kw + self.B * self.Cout * self.Lout) * e
                     + self.Cout * 4)


# A long-sequence fp32 convolution with "same" padding, a channel-heavy bf16 one (even
# dilation), and a strided one that takes the general path.
CONV_WORKLOADS = {
    "v1": ConvWorkload("v1", 21, F32, 16, 64, 65536, 128, 3, 1, 1, 1, ACT_RELU),
    "v2": ConvWorkload("v2", 22, BF16, 8, 256, 16384, 256, 5, 1, 4, 2, ACT_SILU),
    "v3": ConvWorkload("v3", 23, F32, 4, 48, 32768, 64, 5, 2, 2, 1, ACT_NONE),
}


def make_conv_inputs(cw: ConvWorkload, salt: int = 0):
    """(x [B, Cin, L], w [Cout, Cin, Kw], bias [Cout]): x uniform in [-1, 1) (one seeded block of
    2**24 values repeated when the tensor is larger), w normal with standard deviation
    1/sqrt(Cin Kw), bias normal 0.1.  float32, or uint16 bf16 bit patterns for x and w."""
    n = cw.B * cw.Cin * cw.L
    block = uniform(tensor_seed(cw.index, 1, salt), min(n, _REDUCE_BLOCK), -1.0, 1.0)
    x = np.tile(block, (n + block.size - 1) // block.size)[:n].reshape(cw.B, cw.Cin, cw.L)
    w = normal(tensor_seed(cw.index, 2, salt), cw.Cout * cw.Cin * cw.Kw, _inv_sqrt(cw.Cin * cw.Kw))
    w = w.reshape(cw.Cout, cw.Cin, cw.Kw)
    bias = normal(tensor_seed(cw.index, 3, salt), cw.Cout, 0.1)
    if cw.dtype == BF16:
        x, w = f32_to_bf16_bits(x), f32_to_bf16_bits(w)
    return x, w, bias
