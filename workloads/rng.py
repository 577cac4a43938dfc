"""Counter-based random numbers for the synthetic inputs.

A stateless splitmix64 finaliser over (seed, stream, counter) so that the same
(seed, stream, counter) gives the same 64-bit word on any device and in any
batch split.  Everything is written with int64 torch ops (two's-complement
wrap-around multiply, logical shifts emulated with a mask) so a CPU tensor and
a GPU tensor hold identical bits.  This module holds no contraction
arithmetic: it only makes inputs.
"""
import math
import torch

_MASK64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB


def _s64(x):
    """Python int (mod 2**64) -> the signed value with the same bit pattern."""
    x &= _MASK64
    return x - (1 << 64) if x >> 63 else x


def _lsr(x, s):
    """Logical shift right of an int64 tensor."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix_int(z):
    z &= _MASK64
    z = ((z ^ (z >> 30)) * _M1) & _MASK64
    z = ((z ^ (z >> 27)) * _M2) & _MASK64
    return z ^ (z >> 31)


def stream_key(seed, stream):
    """One 64-bit key per (seed, stream-name); stream is a short string."""
    h = _mix_int(seed * _GOLDEN + 0x1234567)
    for ch in stream.encode():
        h = _mix_int(h ^ (ch * _GOLDEN))
    return h


def bits64(seed, stream, start, count, device="cpu"):
    """count 64-bit words for counters start..start+count-1 (int64 bit patterns)."""
    key = stream_key(seed, stream)
    ctr = torch.arange(start, start + count, dtype=torch.int64, device=device)
    z = ctr * _s64(_GOLDEN) + _s64(key)
    z = (z ^ _lsr(z, 30)) * _s64(_M1)
    z = (z ^ _lsr(z, 27)) * _s64(_M2)
    return z ^ _lsr(z, 31)


def uniform01(seed, stream, start, count, device="cpu"):
    """fp64 in [0,1) with 53 random bits."""
    b = _lsr(bits64(seed, stream, start, count, device), 11)
    return b.to(torch.float64) * (1.0 / (1 << 53))


def uniform_int(seed, stream, start, count, n, device="cpu"):
    """Integers in [0,n) (n < 2**31): floor(u*n) of a 53-bit uniform."""
    u = uniform01(seed, stream, start, count, device)
    return torch.clamp((u * n).to(torch.int64), max=n - 1)


def normal(seed, stream, start, count, device="cpu"):
    """N(0,1) by Box-Muller from two uniforms per value."""
    u1 = uniform01(seed, stream + "/a", start, count, device)
    u2 = uniform01(seed, stream + "/b", start, count, device)
    r = torch.sqrt(-2.0 * torch.log(1.0 - u1))     # 1-u1 in (0,1]
    return r * torch.cos((2.0 * math.pi) * u2)


def permutation(seed, stream, n, device="cpu"):
    """A seeded permutation of 0..n-1: order of n distinct-by-construction keys."""
    keys = _lsr(bits64(seed, stream, 0, n, device), 1)           # non-negative
    # ties are broken by position (stable sort), so the result is well defined
    return torch.sort(keys, stable=True).indices
