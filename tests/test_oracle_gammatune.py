"""Pins for oracle.gammatune: hand-worked trajectories, closed forms, invariants
(GammaTune section: eq. adaptive expansion, eq. adaptive window estimation, Algorithm 1)."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import gammatune as gt

GOLD = os.path.join(os.path.dirname(__file__), "golden", "gammatune_trajectories.txt")


def _cases():
    out = []
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, eta, script, gammas, gbars = [x.strip() for x in line.split("|")]
        script = [10**9 if t == "inf" else int(t) for t in script.split()]
        out.append((name, float(eta), script, [int(g) for g in gammas.split()], [float(g) for g in gbars.split()]))
    return out


@pytest.mark.parametrize("name,eta,script,gammas,gbars", _cases(), ids=[c[0] for c in _cases()])
def test_worked_trajectories(name, eta, script, gammas, gbars):
    c = gt.Controller(gt.Params(eta=eta, delta=1, gamma_min=1, gamma_max=8), 4)
    got_g, got_bar = [], []
    for a in script:
        A = min(a, c.gamma)
        got_g.append(c.update(A))
        got_bar.append(c.gamma_bar)
    assert got_g == gammas
    assert got_bar[: len(gbars)] == gbars  # dyadic values: exact in double


def test_closed_form_constant_acceptance():
    # A = 2 < gamma throughout: gamma_bar_n = 2 + (4 - 2) * 0.75**n, never clamped
    c = gt.Controller(gt.Params(eta=0.25, delta=1, gamma_min=1, gamma_max=8), 4)
    for n in range(1, 30):
        c.update(2)
        assert c.gamma_bar == pytest.approx(2 + 2 * 0.75**n, rel=1e-14)
        assert c.gamma == math.ceil(c.gamma_bar)
    assert c.gamma == 3


def test_closed_form_all_reject():
    c = gt.Controller(gt.Params(eta=0.25, delta=1, gamma_min=1, gamma_max=8), 8)
    for n in range(1, 20):
        c.update(0)
        assert c.gamma_bar == pytest.approx(max(1.0, 8 * 0.75**n), rel=1e-14)
    assert c.gamma == 1


def test_all_accept_reaches_gamma_max_and_is_monotone():
    for eta in (0.1, 0.25, 0.5, 0.9):
        c = gt.Controller(gt.Params(eta=eta, delta=1, gamma_min=1, gamma_max=16), 1)
        prev = c.gamma
        for _ in range(400):
            g = c.update(c.gamma)
            assert g >= prev
            prev = g
        assert c.gamma == 16 and c.gamma_bar == 16.0


def test_literal_reading_never_grows():
    c = gt.Controller(gt.Params(eta=0.25, delta=1, gamma_min=1, gamma_max=8, reading=gt.LITERAL), 4)
    for _ in range(50):
        assert c.update(c.gamma) == 4


def test_short_term_reading():
    c = gt.Controller(gt.Params(eta=0.25, delta=2, gamma_min=1, gamma_max=8, reading=gt.SHORT_TERM), 4)
    assert c.update(4) == 6 and c.gamma_bar == 4.0  # jump by delta, EMA on raw A
    assert c.update(3) == 4 and c.gamma_bar == 3.75
    assert c.update(4) == 6
    assert c.update(6) == 8
    assert c.update(8) == 8  # clamped


def test_bounds_and_exact_rational_agreement():
    # random scripts; an exact-rational replay of the recurrence must give the same integers,
    # and gamma_bar must stay inside [gamma_min, gamma_max]
    rng = np.random.default_rng(0)
    for trial in range(200):
        gmin = int(rng.integers(1, 4))
        gmax = int(rng.integers(gmin, 20))
        delta = int(rng.integers(0, 4))
        eta_f = Fraction(int(rng.integers(0, 17)), 16)
        g0 = int(rng.integers(gmin, gmax + 1))
        c = gt.Controller(gt.Params(eta=float(eta_f), delta=delta, gamma_min=gmin, gamma_max=gmax), g0)
        bar, gamma = Fraction(g0), g0
        for _ in range(60):
            A = int(rng.integers(0, gamma + 1))
            a_eff = A + delta if A == gamma else A
            bar = min(Fraction(gmax), max(Fraction(gmin), (1 - eta_f) * bar + eta_f * a_eff))
            gamma = math.ceil(bar)
            got = c.update(A)
            assert gmin <= c.gamma_bar <= gmax
            # doubles drift from the rationals after many steps; the integer must still agree
            # unless the rational sits within rounding distance of an integer
            if abs(bar - round(bar)) > Fraction(1, 10**9) or bar == round(bar):
                assert got == gamma
            bar = Fraction(c.gamma_bar)  # re-anchor so the comparison stays step-local
            gamma = got


def test_early_stop_step_never_expands():
    # GammaTune+: drafted < gamma; A == drafted is not "A == gamma"
    c = gt.Controller(gt.Params(eta=0.25, delta=1, gamma_min=1, gamma_max=8), 4)
    g = c.update(2, 2)
    assert c.gamma_bar == 3.5 and g == 4


def test_input_validation():
    with pytest.raises(ValueError):
        gt.Controller(gt.Params(eta=1.5), 4)
    with pytest.raises(ValueError):
        gt.Controller(gt.Params(gamma_min=0), 4)
    c = gt.Controller(gt.Params(), 4)
    with pytest.raises(ValueError):
        c.update(5)
    with pytest.raises(ValueError):
        c.update(-1)
    with pytest.raises(ValueError):
        c.update(3, 2)
    # gamma0 is clamped into range
    assert gt.Controller(gt.Params(gamma_min=2, gamma_max=5), 9).gamma == 5
