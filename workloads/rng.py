"""Counter-based random numbers: splitmix64 -> uniform(0,1) -> Box-Muller.

Every value is a pure function of (seed, stream, index), so any slice of a
tensor can be regenerated on its own and the same call gives the same bits on
the CPU and on the GPU up to the last ulp of log/cos before the final cast.
Callers that need identical bytes on both sides generate once and copy.

torch has no uint64 arithmetic; int64 with wrap-around multiply/add and an
emulated logical shift gives the same bit patterns.
"""
from __future__ import annotations

import math
import torch

_MASK64 = (1 << 64) - 1


def _s64(x: int) -> int:
    """Reinterpret an unsigned 64-bit constant as a signed Python int."""
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


_GAMMA = _s64(0x9E3779B97F4A7C15)
_M1 = _s64(0xBF58476D1CE4E5B9)
_M2 = _s64(0x94D049BB133111EB)


def _lshr(z: torch.Tensor, n: int) -> torch.Tensor:
    return (z >> n) & ((1 << (64 - n)) - 1)


def _mix(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lshr(z, 30)) * _M1
    z = (z ^ _lshr(z, 27)) * _M2
    return z ^ _lshr(z, 31)


def _mix_int(z: int) -> int:
    z &= _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def _key(seed: int, stream: int) -> int:
    return _mix_int(_mix_int(seed + 0x9E3779B97F4A7C15) ^ (stream * 0xD1342543DE82EF95))


def _bits(seed: int, stream: int, start: int, count: int, device) -> torch.Tensor:
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return _mix(idx * _GAMMA + _s64(_key(seed, stream)))


def uniform01(seed: int, stream: int, n: int, device="cpu", start: int = 0) -> torch.Tensor:
    """n float64 values in the open interval (0,1), indices start..start+n-1."""
    b = _lshr(_bits(seed, stream, start, n, device), 11)      # top 53 bits
    return (b.to(torch.float64) + 0.5) * (1.0 / 9007199254740992.0)


_CHUNK = 1 << 24


def _fill(fn, n: int, dtype, device) -> torch.Tensor:
    out = torch.empty(n, dtype=dtype, device=device)
    for s in range(0, n, _CHUNK):
        c = min(_CHUNK, n - s)
        out[s:s + c] = fn(s, c).to(dtype)
    return out


def normal(seed: int, stream: int, shape, std: float = 1.0, dtype=torch.float32,
           device="cpu") -> torch.Tensor:
    """N(0, std^2) by Box-Muller in fp64 (cosine branch; element i uses
    uniforms 2i and 2i+1), then cast to dtype (round-to-nearest-even)."""
    n = int(math.prod(shape))

    def chunk(s, c):
        u = uniform01(seed, stream, 2 * c, device, start=2 * s).view(c, 2)
        return std * torch.sqrt(-2.0 * torch.log(u[:, 0])) * torch.cos(2.0 * math.pi * u[:, 1])

    return _fill(chunk, n, dtype, device).view(*shape)


def uniform_sym(seed: int, stream: int, shape, bound: float, dtype=torch.float32,
                device="cpu") -> torch.Tensor:
    """U(-bound, bound), cast to dtype."""
    n = int(math.prod(shape))

    def chunk(s, c):
        return (2.0 * uniform01(seed, stream, c, device, start=s) - 1.0) * bound

    return _fill(chunk, n, dtype, device).view(*shape)
