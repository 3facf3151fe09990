"""Counter-based SplitMix64 streams.

Element ``i`` of the stream with seed ``s`` is ``mix(s + (i + 1) * GAMMA)`` where ``mix`` is the
SplitMix64 finaliser (Steele, Lea, Flood 2014).  Because each element depends only on ``(s, i)``,
any slice of a tensor can be regenerated on its own, on the host (numpy, unsigned 64-bit, the
authoritative definition) or on a GPU (torch int64, wrap-around arithmetic gives the same bits).
"""
from __future__ import annotations

import numpy as np

GAMMA = 0x9E3779B97F4A7C15
MIX1 = 0xBF58476D1CE4E5B9
MIX2 = 0x94D049BB133111EB
_MASK64 = (1 << 64) - 1


def splitmix64(seed: int, start: int, count: int) -> np.ndarray:
    """uint64 stream elements ``start .. start+count-1`` for ``seed``."""
    with np.errstate(over="ignore"):
        i = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        z = np.uint64(seed & _MASK64) + i * np.uint64(GAMMA)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(MIX1)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(MIX2)
        z = z ^ (z >> np.uint64(31))
    return z


def uniform01(seed: int, start: int, count: int) -> np.ndarray:
    """float64 in [0, 1): the top 53 bits of each stream element times 2**-53 (exact)."""
    return (splitmix64(seed, start, count) >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)


def uniform_codes(seed: int, count: int, bits: int, start: int = 0) -> np.ndarray:
    """uint8 codes uniform in [0, 2**bits): the top ``bits`` bits of each stream element."""
    return (splitmix64(seed, start, count) >> np.uint64(64 - bits)).astype(np.uint8)


def uniform_fp16(seed: int, count: int, lo: float, hi: float) -> np.ndarray:
    """U(lo, hi) drawn in float64, then rounded to nearest-even binary16."""
    return (lo + (hi - lo) * uniform01(seed, 0, count)).astype(np.float16)


def normal_fp16(seed: int, count: int, scale: np.ndarray | float = 1.0) -> np.ndarray:
    """N(0, 1) by Box-Muller in float64 (element i uses uniforms 2i and 2i+1), times ``scale``,
    then rounded to nearest-even binary16."""
    u = uniform01(seed, 0, 2 * count)
    u1 = 1.0 - u[0::2]  # (0, 1]: keeps the logarithm finite
    u2 = u[1::2]
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return (z * scale).astype(np.float16)


def _signed(c: int) -> int:
    return c - (1 << 64) if c >= (1 << 63) else c


def uniform_codes_torch(seed: int, count: int, bits: int, device, start: int = 0, chunk: int = 1 << 26):
    """Same codes as :func:`uniform_codes`, produced with torch int64 arithmetic on ``device``.

    Two's-complement wrap-around of int64 multiply/add gives the same bit pattern as the unsigned
    definition; the arithmetic right shifts are masked to make them logical.
    """
    import torch

    out = torch.empty(count, dtype=torch.uint8, device=device)
    g, m1, m2 = _signed(GAMMA), _signed(MIX1), _signed(MIX2)
    s = _signed(seed & _MASK64)

    def lsr(x, n):
        return (x >> n) & ((1 << (64 - n)) - 1)

    for lo in range(0, count, chunk):
        n = min(chunk, count - lo)
        i = torch.arange(start + lo + 1, start + lo + n + 1, dtype=torch.int64, device=device)
        z = i * g + s
        z = (z ^ lsr(z, 30)) * m1
        z = (z ^ lsr(z, 27)) * m2
        z = z ^ lsr(z, 31)
        out[lo:lo + n] = lsr(z, 64 - bits).to(torch.uint8)
    return out
