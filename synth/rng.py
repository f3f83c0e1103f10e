"""Counter-based, integer-defined random inputs (torch, any device).

Every value is a pure function of (seed, stream id, step, worker, element
index), so any slice can be produced anywhere (CPU for the oracle, HBM for the
GPU path, one sampled element at a time for full-size checks) and is the same
bits everywhere.  The uniform source is the SplitMix64 output function (Steele,
Lea, Flood 2014): output number n of a stream with state ``base`` is
``mix(base + (n+1)*GAMMA)``.  Only 64-bit integer arithmetic, exact int->float
conversion and single IEEE multiplies are used for the normal variates, so CPU
and GPU torch agree bit for bit.
"""
from __future__ import annotations

import math
from typing import Optional

import torch

MASK64 = (1 << 64) - 1
GAMMA = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB

# stream ids
STREAM_PARAM = 1
STREAM_GRAD = 2
STREAM_LAYOUT = 3
STREAM_ARRIVAL = 4

BASE_SEED = 20250713


def _s64(x: int) -> int:
    """Two's-complement int64 value of a 64-bit pattern."""
    x &= MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


def splitmix64_scalar(x: int) -> int:
    """SplitMix64 output function on a Python int (64-bit wrap-around)."""
    x &= MASK64
    x = ((x ^ (x >> 30)) * _M1) & MASK64
    x = ((x ^ (x >> 27)) * _M2) & MASK64
    return x ^ (x >> 31)


def stream_base(seed: int, stream: int, a: int = 0, b: int = 0) -> int:
    """Derive the state of one independent stream from (seed, stream, a, b)."""
    h = splitmix64_scalar(seed + GAMMA)
    h = splitmix64_scalar(h ^ ((stream + 1) * GAMMA))
    h = splitmix64_scalar(h ^ ((a + 1) * _M1))
    h = splitmix64_scalar(h ^ ((b + 1) * _M2))
    return h


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of int64 bit patterns."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(x: torch.Tensor) -> torch.Tensor:
    x = (x ^ _lsr(x, 30)) * _s64(_M1)
    x = (x ^ _lsr(x, 27)) * _s64(_M2)
    return x ^ _lsr(x, 31)


def uniform_u64(base: int, counter: torch.Tensor) -> torch.Tensor:
    """64 random bits (as int64 patterns) for each int64 ``counter`` >= 0."""
    return _mix((counter + 1) * _s64(GAMMA) + _s64(base))


_IH_MEAN = 8 * 32767.5          # exact: 262140
_IH_STD = math.sqrt(8.0 * (65536.0 ** 2 - 1.0) / 12.0)


def _irwin_hall8(base: int, idx: torch.Tensor, slot: int, nslots: int) -> torch.Tensor:
    """Centred sum of eight 16-bit uniforms (exact small integers, int64)."""
    c = idx * (2 * nslots) + 2 * slot
    s = torch.zeros_like(idx)
    for k in range(2):
        u = uniform_u64(base, c + k)
        for j in range(4):
            s = s + (_lsr(u, 16 * j) & 0xFFFF)
    return s - int(_IH_MEAN)


def normal_f32(base: int, idx: torch.Tensor, sigma: float, slot: int = 0, nslots: int = 1) -> torch.Tensor:
    """~N(0, sigma^2) float32: an 8-term Irwin-Hall sum scaled by one IEEE multiply.

    The integer sum is below 2**20 in magnitude, so its float32 conversion is
    exact; the result is (int) * float32(sigma / std).  Tails end near 4.9 sigma.
    """
    s = _irwin_hall8(base, idx, slot, nslots)
    scale = torch.tensor(sigma / _IH_STD, dtype=torch.float32, device=idx.device)
    return s.to(torch.float32) * scale


def student_t3_f32(base: int, idx: torch.Tensor, scale: float) -> torch.Tensor:
    """scale * Student-t(3): z0 / sqrt((z1^2+z2^2+z3^2)/3) from four unit normals.

    Evaluated in float64 (IEEE +,*,/,sqrt only, identical on CPU and GPU), the
    denominator is clamped at 1e-3, and the product is rounded once to float32.
    """
    z = [(_irwin_hall8(base, idx, k, 4).to(torch.float64)) * (1.0 / _IH_STD) for k in range(4)]
    den = torch.sqrt((z[1] * z[1] + z[2] * z[2] + z[3] * z[3]) / 3.0).clamp_min(1e-3)
    return ((z[0] / den) * scale).to(torch.float32)


def f32_to_bf16_bits(x: torch.Tensor) -> torch.Tensor:
    """Round-to-nearest-even float32 -> bfloat16 bit patterns (int16), finite inputs."""
    b = x.contiguous().view(torch.int32).to(torch.int64) & 0xFFFFFFFF
    b = b + 0x7FFF + ((b >> 16) & 1)
    hi = (b >> 16) & 0xFFFF
    hi = torch.where(hi >= 0x8000, hi - 0x10000, hi)
    return hi.to(torch.int16)


def _periodic(idx: torch.Tensor, period: Optional[int]) -> torch.Tensor:
    return idx if not period else idx % int(period)


def grad_values(seed: int, step: int, worker: int, idx: torch.Tensor, dist: str, sigma: float,
                dtype: str, period: Optional[int] = None) -> torch.Tensor:
    """Gradient of ``worker`` at ``step`` for logical element indices ``idx`` (int64).

    dist: "normal" -> N(0, sigma^2); "t3" -> sigma * Student-t(3).
    dtype: "f32" -> float32 tensor; "bf16" -> int16 tensor of bfloat16 bit patterns.
    period: if set, element e takes the value of element e mod period (a tiled
    input whose global statistics follow from one tile; used at full model size).
    """
    base = stream_base(seed, STREAM_GRAD, step, worker)
    j = _periodic(idx, period)
    if dist == "normal":
        x = normal_f32(base, j, sigma)
    elif dist == "t3":
        x = student_t3_f32(base, j, sigma)
    else:
        raise ValueError(dist)
    if dtype == "f32":
        return x
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


def param_values(seed: int, idx: torch.Tensor, sigma: float = 0.02, period: Optional[int] = None) -> torch.Tensor:
    """Initial parameters ~N(0, sigma^2) (float32) at logical element indices ``idx``."""
    base = stream_base(seed, STREAM_PARAM)
    return normal_f32(base, _periodic(idx, period), sigma)


def tiled(tile: torch.Tensor, idx: torch.Tensor) -> torch.Tensor:
    """Values of a periodic input at indices ``idx`` given one period ``tile`` (= values at 0..period-1)."""
    return tile[idx % tile.numel()]


def arrival_order(seed: int, step: int, num_buckets: int) -> list:
    """Seeded Fisher-Yates shuffle of bucket ids for one step."""
    base = stream_base(seed, STREAM_ARRIVAL, step)
    order = list(range(num_buckets))
    for i in range(num_buckets - 1, 0, -1):
        r = splitmix64_scalar(base + (i + 1) * GAMMA) % (i + 1)
        order[i], order[r] = order[r], order[i]
    return order
