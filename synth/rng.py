"""Counter-based random numbers for the synthetic workloads.

Every draw is a pure function of (seed, stream, index), so an input tensor is the same
whatever device or chunking produced it.  The generator is the public-domain splitmix64
finaliser applied to a 64-bit counter; it is written with torch int64 ops (two's-complement
wrap-around arithmetic), so it runs unchanged on the CPU and on a GPU.

This module holds no arithmetic of the GCN method: it only makes inputs.
"""
from __future__ import annotations

import math

import torch

_MASK64 = (1 << 64) - 1


def _s64(v: int) -> int:
    """Reinterpret an unsigned 64-bit constant as the signed value torch stores."""
    v &= _MASK64
    return v - (1 << 64) if v >= (1 << 63) else v


_GOLDEN = _s64(0x9E3779B97F4A7C15)
_C1 = _s64(0xBF58476D1CE4E5B9)
_C2 = _s64(0x94D049BB133111EB)


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of int64 viewed as u64."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def mix64(counter: torch.Tensor) -> torch.Tensor:
    """splitmix64 output function of an int64 counter tensor (wrapping u64 arithmetic)."""
    z = counter + _GOLDEN
    z = (z ^ _lsr(z, 30)) * _C1
    z = (z ^ _lsr(z, 27)) * _C2
    return z ^ _lsr(z, 31)


def stream_base(seed: int, stream: int) -> int:
    """Signed-int64 start counter of a (seed, stream) pair."""
    return _s64((seed ^ ((stream * 0x9E3779B97F4A7C15) & _MASK64)) & _MASK64)


def bits(seed: int, stream: int, index: torch.Tensor) -> torch.Tensor:
    """64 random bits per element of ``index`` (int64 tensor)."""
    return mix64(index + stream_base(seed, stream))


def uniform(seed: int, stream: int, index: torch.Tensor) -> torch.Tensor:
    """float64 uniforms in [0, 1): top 53 bits of the draw."""
    return _lsr(bits(seed, stream, index), 11).to(torch.float64) * (1.0 / (1 << 53))


def normal(seed: int, stream: int, index: torch.Tensor) -> torch.Tensor:
    """float64 standard normals by Box-Muller on counters 2*index and 2*index+1."""
    u1 = uniform(seed, stream, 2 * index)
    u2 = uniform(seed, stream, 2 * index + 1)
    r = torch.sqrt(-2.0 * torch.log1p(-u1))  # 1-u1 in (0,1]: log never sees 0
    return r * torch.cos((2.0 * math.pi) * u2)


def arange64(n: int, device, start: int = 0) -> torch.Tensor:
    return torch.arange(start, start + n, dtype=torch.int64, device=device)
