"""Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
as 1, 2, 3", SC'11), written from the published round function.

Test infrastructure only (see oracle/__init__.py).

One round maps (c0, c1, c2, c3) with round key (k0, k1) to
    (hi(M1*c2) ^ c1 ^ k0,  lo(M1*c2),  hi(M0*c0) ^ c3 ^ k1,  lo(M0*c0))
with M0 = 0xD2511F53, M1 = 0xCD9E8D57; the key is bumped by the Weyl
constants (0x9E3779B9, 0xBB67AE85) between rounds; ten rounds.

The speculative-decoding step draws its uniforms from
    counter = (s, i, purpose, b),  key = (seed & 0xffffffff, seed >> 32)
with s = speculative-step ordinal, i = row inside the step (1-based),
b = sequence index, purpose one of DRAFT/ACCEPT/RESID/BONUS; the forced
acceptance landscape uses counter = (g, 0, FORCED, b) with g the absolute
index of the generated token.  u = (word0 >> 8) * 2**-24, so u is in [0, 1).
"""
from __future__ import annotations

import numpy as np

M0 = 0xD2511F53
M1 = 0xCD9E8D57
W0 = 0x9E3779B9
W1 = 0xBB67AE85
MASK = 0xFFFFFFFF

DRAFT, ACCEPT, RESID, BONUS, FORCED = 0, 1, 2, 3, 4


def philox4x32_10(counter, key):
    """Scalar version on Python ints. counter: 4 words, key: 2 words."""
    c0, c1, c2, c3 = (int(x) & MASK for x in counter)
    k0, k1 = (int(x) & MASK for x in key)
    for _ in range(10):
        p0 = M0 * c0
        p1 = M1 * c2
        c0, c1, c2, c3 = (
            ((p1 >> 32) ^ c1 ^ k0) & MASK,
            p1 & MASK,
            ((p0 >> 32) ^ c3 ^ k1) & MASK,
            p0 & MASK,
        )
        k0 = (k0 + W0) & MASK
        k1 = (k1 + W1) & MASK
    return c0, c1, c2, c3


def philox4x32_10_array(counters: np.ndarray, key) -> np.ndarray:
    """Vectorised over rows of `counters` ([n, 4] unsigned), same key for all."""
    c = np.asarray(counters, dtype=np.uint64) & np.uint64(MASK)
    c0, c1, c2, c3 = (c[:, j].copy() for j in range(4))
    k0 = np.uint64(int(key[0]) & MASK)
    k1 = np.uint64(int(key[1]) & MASK)
    m = np.uint64(MASK)
    sh = np.uint64(32)
    for _ in range(10):
        p0 = np.uint64(M0) * c0
        p1 = np.uint64(M1) * c2
        n0 = ((p1 >> sh) ^ c1 ^ k0) & m
        n1 = p1 & m
        n2 = ((p0 >> sh) ^ c3 ^ k1) & m
        n3 = p0 & m
        c0, c1, c2, c3 = n0, n1, n2, n3
        k0 = (k0 + np.uint64(W0)) & m
        k1 = (k1 + np.uint64(W1)) & m
    return np.stack([c0, c1, c2, c3], axis=1).astype(np.uint32)


def seed_key(seed: int):
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    return seed & MASK, seed >> 32


def word_to_uniform(word0: int) -> float:
    """24-bit uniform in [0, 1): exactly representable in fp32 and fp64."""
    return float(int(word0) >> 8) * (1.0 / 16777216.0)


def uniform(seed: int, s: int, i: int, purpose: int, b: int) -> float:
    w = philox4x32_10((s, i, purpose, b), seed_key(seed))
    return word_to_uniform(w[0])


def forced_uniform(seed: int, g: int, b: int) -> float:
    return uniform(seed, g, 0, FORCED, b)
