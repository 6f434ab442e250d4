"""GammaTune speculation-length controller (GammaTune section; eq. "adaptive
expansion", eq. "adaptive window estimation", Algorithm 1) in IEEE double.

Test infrastructure only (see oracle/__init__.py).

State: gamma_bar (the smoothed window, a double) and gamma (the integer
length used for the next step).  One update consumes A, the number of
accepted draft tokens of the step just finished (0 <= A <= gamma; the
bonus / resampled token is not counted).

Readings of Algorithm 1
-----------------------
As printed, the expansion branch assigns gamma <- A + delta and the last
statement overwrites gamma <- ceil(gamma_bar), so the branch has no effect
and, because A <= gamma = ceil(gamma_bar), the window can never grow; this
contradicts the surrounding text, which applies the offset delta to A and
states that the window expands in easy regimes.

  EXPAND_A (default)  the offset is applied to the observation:
        A_eff = A + delta if A == gamma else A
        gamma_bar <- min(gmax, max(gmin, (1-eta)*gamma_bar + eta*A_eff))
        gamma <- ceil(gamma_bar)
  LITERAL             the statements exactly as printed (EMA on raw A).
  SHORT_TERM          EMA on raw A; the returned gamma is gamma + delta
                      (clamped) right after a fully accepted step, else
                      ceil(gamma_bar).

GammaTune+ (confidence-guided early stopping) does not change the update:
the test "A == gamma" compares against the planned gamma, so a step that
stopped drafting early (drafted < gamma) never triggers expansion and pulls
gamma_bar towards the small A it produced.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

EXPAND_A, LITERAL, SHORT_TERM = 0, 1, 2


@dataclass
class Params:
    eta: float = 0.25
    delta: int = 1
    gamma_min: int = 1
    gamma_max: int = 8
    reading: int = EXPAND_A


class Controller:
    def __init__(self, params: Params, gamma0: int):
        if not (0.0 <= params.eta <= 1.0):
            raise ValueError("eta outside [0, 1]")
        if params.gamma_min < 1 or params.gamma_max < params.gamma_min:
            raise ValueError("bad gamma range")
        if params.delta < 0:
            raise ValueError("delta < 0")
        if params.reading not in (EXPAND_A, LITERAL, SHORT_TERM):
            raise ValueError("unknown reading")
        self.p = params
        g = min(params.gamma_max, max(params.gamma_min, int(gamma0)))
        self.gamma = g
        self.gamma_bar = float(g)

    def update(self, accepted: int, drafted: int | None = None) -> int:
        p = self.p
        a = int(accepted)
        if a < 0 or a > self.gamma:
            raise ValueError("accepted outside [0, gamma]")
        if drafted is not None and not (a <= drafted <= self.gamma):
            raise ValueError("drafted outside [accepted, gamma]")
        full = a == self.gamma
        a_eff = a + p.delta if (full and p.reading == EXPAND_A) else a
        ema = (1.0 - p.eta) * self.gamma_bar + p.eta * float(a_eff)
        self.gamma_bar = min(float(p.gamma_max), max(float(p.gamma_min), ema))
        nxt = int(math.ceil(self.gamma_bar))
        if p.reading == SHORT_TERM and full:
            nxt = min(p.gamma_max, self.gamma + p.delta)
        self.gamma = nxt
        return nxt


class FixedGamma:
    """Constant speculation length (plain speculative decoding)."""

    def __init__(self, gamma: int):
        self.gamma = int(gamma)
        self.gamma_bar = float(gamma)

    def update(self, accepted: int, drafted: int | None = None) -> int:
        return self.gamma
