"""Counter-based random bits on torch int64 tensors.

Every random number drawn for an input is a pure function of (seed, counter),
so a graph or a feature matrix does not depend on the device it is generated
on, on chunking, or on thread count.  The mixer is the published splitmix64
finaliser; int64 arithmetic in torch wraps modulo 2**64 on both CPU and GPU.
"""
from __future__ import annotations

import torch


def _s64(v: int) -> int:
    """Two's-complement reinterpretation of an unsigned 64-bit constant."""
    v &= (1 << 64) - 1
    return v - (1 << 64) if v >= (1 << 63) else v


_GAMMA = _s64(0x9E3779B97F4A7C15)
_M1 = _s64(0xBF58476D1CE4E5B9)
_M2 = _s64(0x94D049BB133111EB)


def _lsr(x: torch.Tensor, k: int) -> torch.Tensor:
    """Logical shift right of int64 (torch's >> is arithmetic)."""
    return (x >> k) & ((1 << (64 - k)) - 1)


def mix64(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 output function applied element-wise to an int64 tensor."""
    z = x + _GAMMA
    z = (z ^ _lsr(z, 30)) * _M1
    z = (z ^ _lsr(z, 27)) * _M2
    return z ^ _lsr(z, 31)


def stream_key(seed: int, stream: int) -> int:
    """A 64-bit key for one named random stream of one seed (host scalar)."""
    t = torch.tensor([_s64(seed * 0x2545F4914F6CDD1D + stream * 0x9E3779B97F4A7C15 + 0x1234567)],
                     dtype=torch.int64)
    return int(mix64(mix64(t))[0])


def hash_counter(key: int, counter: torch.Tensor) -> torch.Tensor:
    """64 random bits per counter value, for a stream key from stream_key()."""
    return mix64(mix64(counter * _M2 + key))


def uniform01(bits: torch.Tensor) -> torch.Tensor:
    """Top 53 bits of each word as a float64 in [0, 1)."""
    return _lsr(bits, 11).to(torch.float64) * (1.0 / (1 << 53))
