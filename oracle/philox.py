"""Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw: "Parallel random numbers:
as easy as 1, 2, 3", SC'11), written from its published definition.  TEST INFRASTRUCTURE ONLY.

The paper names no generator for its epsilon-greedy draws (Section 2.1) or for "sampled randomly
from D"; the reading taken here fixes one counter-based generator that the oracle and the GPU
library each implement on their own:

    key     = (seed & 0xFFFFFFFF, seed >> 32)
    counter = (index, stream_tag, step & 0xFFFFFFFF, step >> 32)
    stream_tag: 1 = epsilon-greedy draw of environment `index` at act step `step`
                2 = replay sample `index` of sample step `step`
"""
from __future__ import annotations

M0 = 0xD2511F53
M1 = 0xCD9E8D57
W0 = 0x9E3779B9
W1 = 0xBB67AE85
MASK32 = 0xFFFFFFFF

TAG_ACT = 1
TAG_SAMPLE = 2


def philox4x32_10(counter, key):
    """counter: 4 ints, key: 2 ints (each < 2**32) -> tuple of 4 ints."""
    c0, c1, c2, c3 = (int(c) & MASK32 for c in counter)
    k0, k1 = (int(k) & MASK32 for k in key)
    for _ in range(10):
        p0 = M0 * c0
        p1 = M1 * c2
        hi0, lo0 = p0 >> 32, p0 & MASK32
        hi1, lo1 = p1 >> 32, p1 & MASK32
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
        k0 = (k0 + W0) & MASK32
        k1 = (k1 + W1) & MASK32
    return c0, c1, c2, c3


def draw(seed: int, tag: int, step: int, index: int):
    """The four 32-bit outputs for (seed, tag, step, index)."""
    key = (seed & MASK32, (seed >> 32) & MASK32)
    ctr = (index & MASK32, tag, step & MASK32, (step >> 32) & MASK32)
    return philox4x32_10(ctr, key)
