"""Counter-based, sliceable, bit-reproducible value source.

value(seed, tensor_id, i) depends only on its three arguments, so a shard that
needs rows r0..r1 of a tensor evaluates just those flat indices.  All
per-element work is 64-bit integer arithmetic on torch tensors (wrapping
multiply, shifts, masks) followed by one table gather: the same on every device.
"""
from __future__ import annotations

import functools
import math

import numpy as np
import torch

_M32 = 0xFFFFFFFF
_M64 = 0xFFFFFFFFFFFFFFFF


def _mix64(x: int) -> int:
    """One avalanche round on a Python int (splitmix64's finaliser constants)."""
    x &= _M64
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & _M64
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & _M64
    x ^= x >> 31
    return x


def stream_key(seed: int, *parts: int) -> tuple[int, int]:
    """Two 32-bit keys naming one tensor's stream: (seed, part0, part1, ...)."""
    h = _mix64(seed ^ 0x9E3779B97F4A7C15)
    for p in parts:
        h = _mix64(h ^ ((int(p) + 0x632BE59BD9B4E019) & _M64))
    return h & _M32, (h >> 32) & _M32


def _avalanche32(x: torch.Tensor) -> torch.Tensor:
    """32-bit multiply-xorshift hash held in int64 lanes (values stay < 2**32).

    The products overflow int64 and wrap; the low 32 bits of a wrapped product
    are still the low 32 bits of the true product, and the mask keeps only those.
    """
    x = x ^ (x >> 16)
    x = (x * 0x7FEB352D) & _M32
    x = x ^ (x >> 15)
    x = (x * 0x846CA68B) & _M32
    x = x ^ (x >> 16)
    return x


def hash_u32(key: tuple[int, int], idx: torch.Tensor) -> torch.Tensor:
    """Uniform 32-bit values (as int64 in [0, 2**32)) for flat indices `idx`.

    `idx` is an int64 tensor with 0 <= idx < 2**40; the high bits beyond 32 are
    folded in before the second round.
    """
    k1, k2 = key
    lo = idx & _M32
    hi = (idx >> 32) & 0xFF
    x = _avalanche32(lo ^ k1)
    x = _avalanche32(((x + k2) & _M32) ^ (hi * 0x9E3779B1 & _M32))
    return x


@functools.lru_cache(maxsize=None)
def normal_table_f64() -> torch.Tensor:
    """z_k = Phi^-1((k + 0.5) / 65536), k = 0..65535, float64, on the CPU."""
    p = (torch.arange(65536, dtype=torch.float64) + 0.5) / 65536.0
    return torch.special.ndtri(p)


@functools.lru_cache(maxsize=64)
def _table_bf16(mean: float, std: float, device: str) -> torch.Tensor:
    t = (mean + std * normal_table_f64()).to(torch.float32).to(torch.bfloat16)
    return t.to(device)


def normal_bf16(key: tuple[int, int], idx: torch.Tensor, std: float, mean: float = 0.0) -> torch.Tensor:
    """bf16 values ~ N(mean, std^2), one per flat index, on idx's device.

    mean + std * z_k is formed in float64 on the CPU once, rounded to float32 and
    then to bf16 (round-to-nearest-even both times); elements only gather from
    that table.
    """
    table = _table_bf16(float(mean), float(std), str(idx.device))
    return table[hash_u32(key, idx) >> 16]


def uniform_int(key: tuple[int, int], n: int, lo: int, hi: int) -> np.ndarray:
    """n integers uniform on [lo, hi], both ends included (host side, int64)."""
    h = hash_u32(key, torch.arange(n, dtype=torch.int64))
    span = hi - lo + 1
    assert 0 < span < (1 << 31)
    return (lo + ((h * span) >> 32)).numpy()


def lognormal_lengths(key: tuple[int, int], n: int, mu: float, sigma: float, cap: int) -> np.ndarray:
    """n integer lengths: clamp(floor(exp(mu + sigma z) + 0.5), 1, cap), host side."""
    h = hash_u32(key, torch.arange(n, dtype=torch.int64))
    z = normal_table_f64()[h >> 16].numpy()
    out = np.empty(n, dtype=np.int64)
    for i in range(n):
        out[i] = min(max(int(math.floor(math.exp(mu + sigma * float(z[i])) + 0.5)), 1), cap)
    return out
