"""Counter-based random numbers: value = f(seed, stream, index).

Every element of every synthetic tensor is a pure function of
``(seed, stream, index)``, so any slice can be produced independently, in any
order, on any device, in chunks of any size.  The integer part (a 64-bit
finaliser of the splitmix family applied to a keyed counter) is bit-identical
on CPU and GPU; the floating-point part (Box-Muller) is evaluated in fp64 and
may differ in the last bit between devices, which is why a buffer is generated
once and then *copied* to whoever needs it.
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


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right on int64 tensors (torch's >> is arithmetic)."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(x: torch.Tensor) -> torch.Tensor:
    x = (x ^ _lsr(x, 30)) * _C1
    x = (x ^ _lsr(x, 27)) * _C2
    return x ^ _lsr(x, 31)


def _mix_int(v: int) -> int:
    v &= _MASK64
    v = ((v ^ (v >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    v = ((v ^ (v >> 27)) * 0x94D049BB133111EB) & _MASK64
    return v ^ (v >> 31)


def _key(seed: int, stream: int) -> int:
    k = _mix_int((seed + 1) * 0x9E3779B97F4A7C15)
    k = _mix_int(k ^ ((stream + 1) * 0xD1B54A32D192ED03))
    return _s64(k)


def _bits(seed: int, stream: int, start: int, count: int, device) -> torch.Tensor:
    """64 hashed bits (as int64) for counters start .. start+count-1."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return _mix(idx * _GOLDEN + _key(seed, stream))


def uniform01(seed: int, stream: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """fp64 uniforms in the open interval (0, 1)."""
    top53 = _lsr(_bits(seed, stream, start, count, device), 11)
    return (top53.to(torch.float64) + 0.5) * (2.0 ** -53)


def normal(seed: int, stream: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """fp64 standard normals; element i uses counters 2i and 2i+1 (Box-Muller)."""
    u = uniform01(seed, stream, 2 * start, 2 * count, device).view(count, 2)
    r = torch.sqrt(-2.0 * torch.log(u[:, 0]))
    return r * torch.cos((2.0 * math.pi) * u[:, 1])


def randint(seed: int, stream: int, start: int, count: int, high: int, device="cpu") -> torch.Tensor:
    """int64 integers uniform in [0, high)."""
    u = uniform01(seed, stream, start, count, device)
    return torch.clamp((u * high).to(torch.int64), max=high - 1)


def stream_key(seed: int, stream: int) -> int:
    """The 64-bit key of (seed, stream) as an unsigned integer: what a consumer that implements this generator
    itself (counter -> hashed bits) needs besides the counter."""
    return _key(seed, stream) & _MASK64


def uniform23(key: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """fp64 uniforms in (0, 1) with 23 random bits each, (n + 0.5) * 2^-23, for counters start .. start+count-1 of
    the stream with the given 64-bit key: values an fp32 holds exactly, so an fp32 consumer sees the same numbers."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    top23 = _lsr(_mix(idx * _GOLDEN + _s64(key)), 41)
    return (top23.to(torch.float64) + 0.5) * (2.0 ** -23)
