"""Counter-based random numbers: value(i) = f(seed, stream, i).

Every element of every synthetic tensor is a pure function of (seed, stream id,
element index), so a tensor can be produced in pieces, on the host or on the
device, and always holds the same integers.  The mixing function is the
SplitMix64 finaliser (Steele, Lea, Flood 2014) applied to a Weyl sequence;
normals come from the Box-Muller transform of two 24-bit uniforms.

All integer work is done on int64 tensors with wrap-around multiplication,
which torch implements identically on CPU and GPU.
"""
from __future__ import annotations

import math
import torch

_MASK32 = (1 << 32) - 1


def _s64(v: int) -> int:
    """Interpret an unsigned 64-bit constant as the int64 with the same bits."""
    v &= (1 << 64) - 1
    return v - (1 << 64) if v >= (1 << 63) else v


_GOLDEN = _s64(0x9E3779B97F4A7C15)
_M1 = _s64(0xBF58476D1CE4E5B9)
_M2 = _s64(0x94D049BB133111EB)


def _lsr(z: torch.Tensor, k: int) -> torch.Tensor:
    """Logical right shift of int64 bit patterns."""
    return (z >> k) & ((1 << (64 - k)) - 1)


def uniform_bits(seed: int, stream: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """64 mixed bits per element for indices start .. start+count-1 (int64 tensor)."""
    i = torch.arange(start, start + count, dtype=torch.int64, device=device)
    z = (i + 1) * _GOLDEN + _s64(seed * 0x2545F4914F6CDD1D + stream * 0xD1B54A32D192ED03)
    z = (z ^ _lsr(z, 30)) * _M1
    z = (z ^ _lsr(z, 27)) * _M2
    z = z ^ _lsr(z, 31)
    return z


def uniform01(seed: int, stream: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """float64 uniforms in [0, 1) with 53 random bits."""
    z = uniform_bits(seed, stream, start, count, device)
    return _lsr(z, 11).to(torch.float64) * (1.0 / (1 << 53))


def normal(seed: int, stream: int, shape, std: float = 1.0, mean: float = 0.0,
           device="cpu", dtype=torch.float32, chunk: int = 1 << 24) -> torch.Tensor:
    """N(mean, std^2) samples of the given shape, element i from counter i."""
    n = int(math.prod(shape)) if len(shape) else 1
    out = torch.empty(n, dtype=dtype, device=device)
    for s in range(0, n, chunk):
        c = min(chunk, n - s)
        z = uniform_bits(seed, stream, s, c, device)
        a = (_lsr(z, 40) & 0xFFFFFF).to(torch.float32)          # top 24 bits
        b = (_lsr(z, 8) & 0xFFFFFF).to(torch.float32)           # next 24 bits
        u1 = (a + 1.0) * (1.0 / 16777216.0)                     # (0, 1]
        u2 = b * (1.0 / 16777216.0)                             # [0, 1)
        g = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)
        out[s:s + c] = (g * std + mean).to(dtype)
    return out.reshape(shape)


def randint(seed: int, stream: int, lo: int, hi: int, count: int, device="cpu") -> torch.Tensor:
    """Integers uniform in [lo, hi] inclusive (int64).  Modulo bias < 2^-40 for the ranges used."""
    z = uniform_bits(seed, stream, 0, count, device)
    span = hi - lo + 1
    return (_lsr(z, 16) % span) + lo


def permutation(seed: int, stream: int, n: int) -> torch.Tensor:
    """A seeded permutation of 0..n-1: argsort of n counter-based keys (ties broken by index)."""
    z = _lsr(uniform_bits(seed, stream, 0, n), 1)
    return torch.sort(z, stable=True).indices
