"""Seeded synthetic KV-cache contents for verify-only sweeps: values N(0, 0.5^2) that bfloat16 holds exactly,
so that a 16-bit cache and a float64 reference start from identical numbers."""
from __future__ import annotations

import numpy as np


def make_kv(n: int, n_kv_heads: int, head_dim: int, seed: int):
    """(k, v): float32 [n, n_kv_heads, head_dim], every value a bfloat16 number."""
    rng = np.random.default_rng(int(seed))

    def one():
        a = (rng.standard_normal((n, n_kv_heads, head_dim)) * 0.5).astype(np.float32)
        bits = a.view(np.uint32)
        bits = (bits + np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
        return bits.view(np.float32)

    return one(), one()
