"""Seeded prompts: uniform-random token ids (stand-in for benchmark prompts, which
are not available offline and are never reconstructed)."""
from __future__ import annotations

import numpy as np


def make_prompts(batch: int, length: int, vocab: int, seed: int) -> np.ndarray:
    """int32 [batch, length], ids uniform in [0, vocab)."""
    rng = np.random.default_rng(int(seed))
    return rng.integers(0, vocab, size=(batch, length), dtype=np.int64).astype(np.int32)
