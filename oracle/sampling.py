"""Sampling rules of speculative sampling (Background section; the rule itself
is the one of the works cited there, Leviathan et al. and Chen et al.):
a draft token x ~ q is kept when u < min(1, p(x)/q(x)); at the first refusal
a replacement is drawn from norm(max(0, p - q)); when every draft token is
kept one more token is drawn from the target's next distribution.

Test infrastructure only (see oracle/__init__.py).  All arithmetic in fp64.

Conventions (fixed here, identical text on the GPU side):
  * p = softmax(logits / T); T == 0 means greedy (argmax, lowest index wins)
  * a token is drawn from non-negative weights w by index-order inverse CDF:
        y = min{ j : w_0 + ... + w_j > u * W },  W = sum(w)
    and, should rounding leave no such j, the last j with w_j > 0
  * the accept test is evaluated as  u * q(x) < p(x)  (same as u < p/q and
    true whenever p >= q because u < 1)
Each decision also reports a margin: how far it is from flipping, used by
the parity tests to tell a real disagreement from a rounding-level one.
"""
from __future__ import annotations

import numpy as np


def argmax_lowest(x: np.ndarray) -> int:
    return int(np.argmax(x))  # numpy returns the first maximal index


def top2_gap(x: np.ndarray) -> float:
    if x.shape[0] < 2:
        return float("inf")
    part = np.partition(x, -2)
    return float(part[-1] - part[-2])


def softmax_T(logits: np.ndarray, T: float) -> np.ndarray:
    z = (np.asarray(logits, dtype=np.float64) - np.max(logits)) / float(T)
    w = np.exp(z)
    return w / w.sum()


def top_probability(logits: np.ndarray, T_eff: float) -> float:
    """max_x softmax(logits / T_eff)(x): the draft's confidence (GammaTune+)."""
    z = (np.asarray(logits, dtype=np.float64) - np.max(logits)) / float(T_eff)
    return float(1.0 / np.exp(z).sum())


def inverse_cdf(w: np.ndarray, u: float):
    """Return (index, margin); margin = distance of u*W to the nearest CDF edge, over W."""
    w = np.asarray(w, dtype=np.float64)
    c = np.cumsum(w)
    W = float(c[-1])
    t = u * W
    j = int(np.searchsorted(c, t, side="right"))  # first j with c[j] > t
    if j >= w.shape[0]:
        nz = np.nonzero(w > 0)[0]
        j = int(nz[-1]) if nz.size else w.shape[0] - 1
        return j, 0.0
    lo = c[j - 1] if j > 0 else 0.0
    margin = min(t - lo, c[j] - t) / W if W > 0 else 0.0
    if j == 0:
        margin = (c[0] - t) / W if W > 0 else 0.0
    return j, float(margin)


def accept_test(p_x: float, q_x: float, u: float):
    """Return (accepted, margin) for u*q < p; margin = |u*q - p| / max(p, q)."""
    lhs = u * q_x
    ok = lhs < p_x
    den = max(p_x, q_x)
    margin = abs(lhs - p_x) / den if den > 0 else 0.0
    return bool(ok), float(margin)


def residual_weights(p: np.ndarray, q: np.ndarray) -> np.ndarray:
    return np.maximum(0.0, np.asarray(p, dtype=np.float64) - np.asarray(q, dtype=np.float64))


def sample_residual(p: np.ndarray, q: np.ndarray, u: float):
    """Draw from norm(max(0, p - q)); falls back to p if the residual mass is not positive."""
    w = residual_weights(p, q)
    if not (w.sum() > 0.0):
        return inverse_cdf(p, u)
    return inverse_cdf(w, u)
