"""Integer-only counter-based random streams (SplitMix64).

Every random input of the test and benchmark workloads is drawn from a
SplitMix64 stream whose seed is derived from (config seed, stream tag), so
that a C++ program and a Python program can regenerate identical inputs.
"""
M64 = (1 << 64) - 1
MASTER_SEED = 250601151


class SplitMix64:
    """Vigna's SplitMix64: state += golden gamma, then a 3-step finaliser."""

    __slots__ = ("s",)

    def __init__(self, seed: int):
        self.s = seed & M64

    def next_u64(self) -> int:
        self.s = (self.s + 0x9E3779B97F4A7C15) & M64
        z = self.s
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
        return z ^ (z >> 31)

    def below(self, n: int) -> int:
        """Uniform-ish integer in [0, n) by modulo (bias accepted, documented)."""
        return self.next_u64() % n


def _fnv1a(data: bytes) -> int:
    h = 0xCBF29CE484222325
    for b in data:
        h = ((h ^ b) * 0x100000001B3) & M64
    return h


def stream(config_seed: int, tag: str) -> SplitMix64:
    """Independent stream for (config seed, tag): seed = mix(seed ^ fnv1a(tag))."""
    return SplitMix64(SplitMix64(config_seed ^ _fnv1a(tag.encode())).next_u64())
