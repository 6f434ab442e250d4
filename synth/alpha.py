"""Forced-acceptance schedules alpha(g), g = index of the generated token.

They stand in for the acceptance landscape of real text (easy / moderate /
difficult regimes of the GammaTune section): a constant rate, or a rate that
alternates between two levels every `period` tokens.
"""
from __future__ import annotations

import numpy as np


def alpha_constant(alpha: float, n: int) -> np.ndarray:
    return np.full(int(n), float(alpha), dtype=np.float32)


def alpha_piecewise(n: int, period: int = 32, hi: float = 0.9, lo: float = 0.3) -> np.ndarray:
    g = np.arange(int(n))
    return np.where((g // period) % 2 == 0, hi, lo).astype(np.float32)
