"""Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw: "Parallel random
numbers: as easy as 1, 2, 3", SC'11), written from the published round function.

Test infrastructure.  The rollout path draws one 32-bit word per (sample, step):
key = (seed low word, seed high word), counter = (sample_id low, sample_id high, step, 0),
and the word used is output word 0.  Pinned by the known-answer vectors distributed with
the authors' reference implementation.
"""
from __future__ import annotations

MASK32 = 0xFFFFFFFF
MULT_A = 0xD2511F53   # multiplies counter word 0
MULT_B = 0xCD9E8D57   # multiplies counter word 2
WEYL_A = 0x9E3779B9   # key word 0 increment per round (golden ratio)
WEYL_B = 0xBB67AE85   # key word 1 increment per round (sqrt(3) - 1)


def philox4x32(counter, key, rounds: int = 10):
    """One block: counter = 4 words, key = 2 words, returns 4 output words."""
    c0, c1, c2, c3 = (int(c) & MASK32 for c in counter)
    k0, k1 = (int(k) & MASK32 for k in key)
    for r in range(rounds):
        if r:
            k0 = (k0 + WEYL_A) & MASK32
            k1 = (k1 + WEYL_B) & MASK32
        p0 = MULT_A * c0
        p1 = MULT_B * c2
        c0, c1, c2, c3 = ((p1 >> 32) ^ c1 ^ k0) & MASK32, p1 & MASK32, \
                         ((p0 >> 32) ^ c3 ^ k1) & MASK32, p0 & MASK32
    return c0, c1, c2, c3


def rollout_uniform(seed: int, sample_id: int, step: int) -> int:
    """The 32-bit word that drives sample `sample_id`'s draw at response position `step`."""
    key = (seed & MASK32, (seed >> 32) & MASK32)
    ctr = (sample_id & MASK32, (sample_id >> 32) & MASK32, step & MASK32, 0)
    return philox4x32(ctr, key)[0]
