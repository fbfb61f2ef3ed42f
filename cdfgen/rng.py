"""Counter-based random numbers built from integer tensor ops only.

Every draw is a pure function of (seed, stream, counter), so a value does not
depend on the device that computed it or on how the counters were batched.
The mixer is the SplitMix64 finaliser (Steele, Lea, Flood 2014), evaluated on
int64 tensors whose arithmetic wraps modulo 2**64.

This module holds input generation only: none of the cache, quantiser,
aggregation or layer arithmetic lives here.
"""
import math

import torch

_M1 = 0xBF58476D1CE4E5B9 - (1 << 64)
_M2 = 0x94D049BB133111EB - (1 << 64)
_GOLD = 0x9E3779B97F4A7C15 - (1 << 64)


def _lsr(x: torch.Tensor, k: int) -> torch.Tensor:
    """Logical shift right of an int64 tensor."""
    return (x >> k) & ((1 << (64 - k)) - 1)


def mix64(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 30)) * _M1
    z = (z ^ _lsr(z, 27)) * _M2
    return z ^ _lsr(z, 31)


def _wrap(v: int) -> int:
    v &= (1 << 64) - 1
    return v - (1 << 64) if v >= (1 << 63) else v


def stream_key(seed: int, stream: int) -> int:
    """Scalar key separating independent streams of one seed."""
    z = _wrap(seed * 0x9E3779B97F4A7C15 + stream * 0xD1B54A32D192ED03 + 0x2545F4914F6CDD1D)
    t = torch.tensor([z], dtype=torch.int64)
    return int(mix64(t).item())


def bits64(seed: int, stream: int, counter: torch.Tensor) -> torch.Tensor:
    """64 random bits per counter value (int64 tensor, any device)."""
    key = stream_key(seed, stream)
    return mix64(counter * _GOLD + key)


def uniform01(seed: int, stream: int, counter: torch.Tensor) -> torch.Tensor:
    """float64 uniform in the open interval (0, 1)."""
    b = _lsr(bits64(seed, stream, counter), 11)
    return (b.to(torch.float64) + 0.5) * (1.0 / (1 << 53))


def normal(seed: int, stream: int, n: int, device="cpu", dtype=torch.float32,
           chunk: int = 1 << 24) -> torch.Tensor:
    """n standard normal draws (Box-Muller on two uniforms per value)."""
    out = torch.empty(n, dtype=dtype, device=device)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        c = torch.arange(s, e, dtype=torch.int64, device=device)
        u1 = uniform01(seed, stream, 2 * c)
        u2 = uniform01(seed, stream, 2 * c + 1)
        z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)
        out[s:e] = z.to(dtype)
    return out


def uniform(seed: int, stream: int, n: int, lo=0.0, hi=1.0, device="cpu",
            dtype=torch.float32) -> torch.Tensor:
    c = torch.arange(n, dtype=torch.int64, device=device)
    return (lo + (hi - lo) * uniform01(seed, stream, c)).to(dtype)
