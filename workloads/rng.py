"""Counter-based random numbers for the synthetic inputs.

Every value is a pure function of (seed, stream, index): a 64-bit integer mix
evaluated with torch int64 arithmetic, so the integer streams are the same on
any device.  This module holds input generation only; nothing of the sampled
SpMM method lives here.
"""
from __future__ import annotations

import math

import torch

_MASK64 = (1 << 64) - 1


def _s64(v: int) -> int:
    """Python int -> the signed 64-bit value with the same bit pattern."""
    v &= _MASK64
    return v - (1 << 64) if v >= (1 << 63) else v


_GOLDEN = _s64(0x9E3779B97F4A7C15)
_MUL1 = _s64(0xBF58476D1CE4E5B9)
_MUL2 = _s64(0x94D049BB133111EB)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 lanes."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 30)) * _MUL1
    z = (z ^ _lsr(z, 27)) * _MUL2
    return z ^ _lsr(z, 31)


def _mix_int(v: int) -> int:
    v &= _MASK64
    v = ((v ^ (v >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    v = ((v ^ (v >> 27)) * 0x94D049BB133111EB) & _MASK64
    return v ^ (v >> 31)


def bits(seed: int, stream: int, n: int, device, start: int = 0) -> torch.Tensor:
    """n pseudo-random int64 bit patterns for counters start .. start+n-1."""
    key = _s64(_mix_int(_mix_int(seed) ^ ((stream + 1) * 0xD1B54A32D192ED03)))
    ctr = torch.arange(start, start + n, dtype=torch.int64, device=device)
    return _mix(ctr * _GOLDEN + key)


def uniform(seed: int, stream: int, n: int, device, start: int = 0) -> torch.Tensor:
    """float64 in [0, 1)."""
    return _lsr(bits(seed, stream, n, device, start), 11).to(torch.float64) * (2.0 ** -53)


def normal(seed: int, stream: int, n: int, device) -> torch.Tensor:
    """float64 standard normal (Box-Muller on two streams)."""
    u1 = 1.0 - uniform(seed, 2 * stream, n, device)          # (0, 1]
    u2 = uniform(seed, 2 * stream + 1, n, device)
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)


def permutation(seed: int, stream: int, n: int, device) -> torch.Tensor:
    """A permutation of 0..n-1 (argsort of random keys; ties broken by index)."""
    return torch.argsort(_lsr(bits(seed, stream, n, device), 1), stable=True)
