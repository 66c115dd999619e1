"""Counter-based random numbers for the seeded synthetic inputs.

Every array is a pure function of (seed, stream, counter): element `c` of stream
`s` is `mix64(key(seed, s) + c * GOLDEN)`.  The mixer is the public splitmix64
finaliser, written with torch int64 ops so the same arrays come out on the host
and on a GPU.  Nothing here knows about tensors, formats or the operations.
"""
from __future__ import annotations

import torch

_M64 = (1 << 64) - 1


def _s64(x: int) -> int:
    """Reinterpret an unsigned 64-bit constant as the signed value torch stores."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


_GOLDEN = _s64(0x9E3779B97F4A7C15)
_C1 = _s64(0xBF58476D1CE4E5B9)
_C2 = _s64(0x94D049BB133111EB)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 (torch's >> is arithmetic)."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def mix64(z: torch.Tensor) -> torch.Tensor:
    """splitmix64 finaliser: a bijection on 64-bit words (int64 in, int64 out)."""
    z = (z ^ _lsr(z, 30)) * _C1
    z = (z ^ _lsr(z, 27)) * _C2
    return z ^ _lsr(z, 31)


def _mix64_int(z: int) -> int:
    z &= _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def stream_key(seed: int, stream: int) -> int:
    """Start value of a stream; distinct (seed, stream) pairs give unrelated streams."""
    return _s64(_mix64_int(_mix64_int(seed) ^ ((stream * 0xD1342543DE82EF95) & _M64)))


def bits64(seed: int, stream: int, n: int, device="cpu", offset: int = 0) -> torch.Tensor:
    """n raw 64-bit words (as int64) for counters offset .. offset+n-1."""
    c = torch.arange(offset, offset + n, dtype=torch.int64, device=device)
    return mix64(c * _GOLDEN + stream_key(seed, stream))


def hash64(keys: torch.Tensor, seed: int, stream: int) -> torch.Tensor:
    """Hash arbitrary int64 keys (used for deterministic thinning and permutations)."""
    return mix64(keys * _GOLDEN + stream_key(seed, stream))


def uniform01(seed: int, stream: int, n: int, device="cpu", offset: int = 0) -> torch.Tensor:
    """float64 in [0, 1): the top 53 bits of each word times 2**-53 (exact)."""
    return _lsr(bits64(seed, stream, n, device, offset), 11).to(torch.float64) * (2.0 ** -53)


def uniform_pm1(seed: int, stream: int, n: int, device="cpu", offset: int = 0) -> torch.Tensor:
    """float64 in [-1, 1)."""
    return uniform01(seed, stream, n, device, offset) * 2.0 - 1.0


def randint(seed: int, stream: int, n: int, high: int, device="cpu", offset: int = 0) -> torch.Tensor:
    """int64 in [0, high): floor(u * high); high < 2**31 keeps it exact in float64."""
    u = uniform01(seed, stream, n, device, offset)
    return torch.clamp((u * float(high)).to(torch.int64), max=high - 1)


def permutation(seed: int, stream: int, n: int, device="cpu") -> torch.Tensor:
    """A seeded permutation of 0..n-1: the argsort of n distinct 64-bit hashes."""
    h = bits64(seed, stream, n, device)
    return torch.argsort(h, stable=True)
