"""Counter-based 64-bit generator used by every seeded synthetic input.

SplitMix64 (Steele, Lea, Flood 2014): a Weyl sequence with a 64-bit finaliser.
Both a sequential form (``SplitMix64``) for host-side workload construction and
a stateless, vectorised form (``mix64``) for pool/weight content are provided.
Nothing here belongs to the KV-reclaim method itself.
"""
from __future__ import annotations

import math

import numpy as np

MASK64 = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15
MUL1 = 0xBF58476D1CE4E5B9
MUL2 = 0x94D049BB133111EB


def mix64_int(z: int) -> int:
    """SplitMix64 finaliser on a Python int (mod 2**64)."""
    z &= MASK64
    z = ((z ^ (z >> 30)) * MUL1) & MASK64
    z = ((z ^ (z >> 27)) * MUL2) & MASK64
    return z ^ (z >> 31)


def mix64(z: np.ndarray) -> np.ndarray:
    """SplitMix64 finaliser on a uint64 array (wrapping arithmetic)."""
    z = z.astype(np.uint64, copy=True)
    z ^= z >> np.uint64(30)
    z *= np.uint64(MUL1)
    z ^= z >> np.uint64(27)
    z *= np.uint64(MUL2)
    z ^= z >> np.uint64(31)
    return z


class SplitMix64:
    """Sequential SplitMix64 stream."""

    def __init__(self, seed: int):
        self.state = seed & MASK64

    def next_u64(self) -> int:
        self.state = (self.state + GOLDEN) & MASK64
        return mix64_int(self.state)

    def below(self, n: int) -> int:
        """Integer in [0, n) by multiply-shift (bias < n / 2**64)."""
        return (self.next_u64() * n) >> 64

    def uniform(self) -> float:
        """Double in [0, 1) with 53 random bits."""
        return (self.next_u64() >> 11) * (1.0 / (1 << 53))

    def randint(self, lo: int, hi: int) -> int:
        """Integer uniform on the closed interval [lo, hi]."""
        return lo + self.below(hi - lo + 1)

    def log_uniform_int(self, lo: int, hi: int) -> int:
        """floor(lo * (hi/lo)**U), clamped to [lo, hi]."""
        v = int(math.floor(lo * math.exp(self.uniform() * math.log(hi / lo))))
        return min(max(v, lo), hi)

    def shuffle(self, n: int) -> list[int]:
        """Fisher-Yates shuffle of range(n)."""
        a = list(range(n))
        for i in range(n - 1, 0, -1):
            j = self.below(i + 1)
            a[i], a[j] = a[j], a[i]
        return a
