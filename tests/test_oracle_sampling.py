"""Pins for oracle.sampling and oracle.spec: the accept / resample law equals the target
distribution (Background section: speculative sampling reproduces target-only sampling)."""
import itertools
import math

import numpy as np
import pytest

from oracle import gammatune as gt
from oracle import philox
from oracle import sampling as S
from oracle import spec


def _lattice(M):
    return (np.arange(M) + 0.5) / M


def _measure_one_token_law(p, q, M):
    """Law of the emitted token when x ~ q is tested against p, every stage measured on a lattice
    through the oracle's own functions.  Each 1-D frequency is within (#edges)/M of the truth."""
    V = len(p)
    us = _lattice(M)
    qhat = np.bincount([S.inverse_cdf(q, u)[0] for u in us], minlength=V) / M
    out = np.zeros(V)
    rej_mass = 0.0
    for x in range(V):
        if qhat[x] == 0:
            continue
        acc = np.mean([S.accept_test(p[x], q[x], u)[0] for u in us])
        out[x] += qhat[x] * acc
        rej_mass += qhat[x] * (1 - acc)
    if rej_mass > 0:
        rhat = np.bincount([S.sample_residual(p, q, u)[0] for u in us], minlength=V) / M
        out += rej_mass * rhat
    return out


@pytest.mark.parametrize("V", [2, 3, 5, 6])
def test_emitted_law_equals_target_brute_force(V):
    rng = np.random.default_rng(V)
    M = 1 << 14
    for _ in range(6):
        p = rng.dirichlet(np.ones(V))
        q = rng.dirichlet(np.ones(V))
        law = _measure_one_token_law(p, q, M)
        assert np.max(np.abs(law - p)) <= 3.0 * (V + 1) / M
        assert abs(law.sum() - 1.0) < 1e-12


def test_identity_min_plus_residual():
    # min(p,q) + (1 - sum min(p,q)) * norm(max(0,p-q)) == p, with the residual law measured
    rng = np.random.default_rng(3)
    M = 1 << 15
    for V in (3, 4, 6):
        p = rng.dirichlet(np.ones(V))
        q = rng.dirichlet(np.ones(V))
        rhat = np.bincount([S.sample_residual(p, q, u)[0] for u in _lattice(M)], minlength=V) / M
        lhs = np.minimum(p, q) + (1 - np.minimum(p, q).sum()) * rhat
        assert np.max(np.abs(lhs - p)) <= (V + 1) / M


def test_edge_cases():
    us = _lattice(256)
    p = np.array([0.2, 0.5, 0.3])
    # p == q: always accepted
    assert all(S.accept_test(p[x], p[x], u)[0] for x in range(3) for u in us)
    # disjoint supports: always rejected, residual == p
    p2 = np.array([0.0, 0.0, 0.4, 0.6])
    q2 = np.array([0.5, 0.5, 0.0, 0.0])
    assert not any(S.accept_test(p2[x], q2[x], u)[0] for x in (0, 1) for u in us)
    r = np.bincount([S.sample_residual(p2, q2, u)[0] for u in _lattice(1000)], minlength=4) / 1000
    assert np.allclose(r, p2, atol=2e-3)
    # q one-hot on a token the target also likes: accepted with prob p(x)
    q3 = np.array([0.0, 1.0, 0.0])
    acc = np.mean([S.accept_test(p[1], q3[1], u)[0] for u in us])
    assert acc == pytest.approx(0.5, abs=1 / 256)
    # inverse CDF: zero-weight tokens are never drawn, u -> 1 picks the last positive weight
    w = np.array([0.0, 1.0, 0.0, 3.0, 0.0])
    drawn = {S.inverse_cdf(w, u)[0] for u in us}
    assert drawn == {1, 3}
    assert S.inverse_cdf(w, 1.0 - 2**-24)[0] == 3
    assert S.inverse_cdf(w, 0.0)[0] == 1
    # argmax ties -> lowest index
    assert S.argmax_lowest(np.array([1.0, 3.0, 3.0, 2.0])) == 1
    # residual with no mass falls back to p
    assert S.sample_residual(p, p, 0.1)[0] == S.inverse_cdf(p, 0.1)[0]


def test_softmax_temperature_and_top_probability():
    l = np.array([0.0, math.log(2.0), math.log(5.0)])
    assert np.allclose(S.softmax_T(l, 1.0), [1 / 8, 2 / 8, 5 / 8])
    assert np.allclose(S.softmax_T(l, 0.5), np.array([1, 4, 25]) / 30.0)
    assert S.top_probability(l, 1.0) == pytest.approx(5 / 8)
    assert S.top_probability(l, 0.5) == pytest.approx(25 / 30)
    assert S.softmax_T(l + 1000.0, 1.0) == pytest.approx(S.softmax_T(l, 1.0))  # shift-safe


class _Tables:
    """Markov toy models: next-token law depends on the last token only; logits = log prob."""

    def __init__(self, P, Q):
        self.P, self.Q = np.asarray(P, float), np.asarray(Q, float)

    def draft_next(self, toks):
        return np.log(self.Q[toks[-1]])

    def target_rows(self, toks, k):
        return np.stack([np.log(self.P[toks[len(toks) - k - 1 + j]]) for j in range(k + 1)])


def _lattice_uniform(coords, dims):
    """uniform(s, i, purpose, b) reading a lattice point chosen per (purpose, row)."""
    def u(s, i, purpose, b):
        key = (purpose, i)
        # RESID and BONUS never occur in the same step: they share one lattice axis
        if purpose in (philox.RESID, philox.BONUS):
            key = ("last", 0)
        return coords[dims.index(key)]
    return u


def test_two_token_step_joint_law_exact():
    # gamma = 2, V = 3, all probabilities in {1/4, 1/2}: every decision edge is a multiple of 1/8,
    # so midpoints of an 8-point lattice integrate every uniform exactly.
    a, b_, c = (0.5, 0.25, 0.25), (0.25, 0.5, 0.25), (0.25, 0.25, 0.5)
    P = [b_, c, a]
    Q = [a, b_, c]
    tm = _Tables(P, Q)
    M = 8
    us = _lattice(M)
    dims = [(philox.DRAFT, 1), (philox.DRAFT, 2), (philox.ACCEPT, 1), (philox.ACCEPT, 2), ("last", 0)]
    cfg = spec.StepConfig(temperature=1.0)
    start = 0
    joint = np.zeros((3, 3))
    first = np.zeros(3)
    acc_hist = np.zeros(3)
    for coords in itertools.product(us, repeat=5):
        r = spec.speculative_step(tm.draft_next, tm.target_rows, [start], 2, 0, 0, cfg, 0,
                                  uniform=_lattice_uniform(coords, dims))
        w = 1.0 / M**5
        e = r.emitted
        first[e[0]] += w
        acc_hist[r.accepted] += w
        if len(e) >= 2:
            joint[e[0], e[1]] += w
        else:  # complete with the target's own conditional
            joint[e[0], :] += w * np.asarray(P[e[0]])
    Pm = np.asarray(P)
    assert np.allclose(first, Pm[start], atol=1e-12)
    want = Pm[start][:, None] * Pm
    assert np.allclose(joint, want, atol=1e-12)
    # acceptance count: P(A >= 1) = sum_x min(p, q)
    assert acc_hist[1] + acc_hist[2] == pytest.approx(np.minimum(Pm[start], np.asarray(Q)[start]).sum(), abs=1e-12)


def test_one_token_step_exact_with_spread_residual():
    # V = 4, residual norm(max(0,p-q)) = (0, 0, 1/4, 3/4): all edges multiples of 1/8
    q = np.array([1 / 2, 1 / 4, 1 / 8, 1 / 8])
    p = np.array([1 / 8, 1 / 8, 1 / 4, 1 / 2])
    tm = _Tables([p] * 4, [q] * 4)
    M = 8
    us = _lattice(M)
    dims = [(philox.DRAFT, 1), (philox.ACCEPT, 1), ("last", 0)]
    cfg = spec.StepConfig(temperature=1.0)
    law = np.zeros(4)
    n_acc = 0.0
    for coords in itertools.product(us, repeat=3):
        r = spec.speculative_step(tm.draft_next, tm.target_rows, [0], 1, 0, 0, cfg, 0,
                                  uniform=_lattice_uniform(coords, dims))
        law[r.emitted[0]] += 1.0 / M**3
        n_acc += r.accepted / M**3
    assert np.allclose(law, p, atol=1e-12)
    assert n_acc == pytest.approx(np.minimum(p, q).sum(), abs=1e-12)


def test_temperature_enters_both_models():
    # with T = 2 the emitted law is softmax(log p / 2), i.e. proportional to sqrt(p)
    q = np.array([1 / 2, 1 / 4, 1 / 8, 1 / 8])
    p = np.array([1 / 8, 1 / 8, 1 / 4, 1 / 2])
    tm = _Tables([p] * 4, [q] * 4)
    rng = np.random.default_rng(5)
    n = 20000
    cnt = np.zeros(4)
    cfg = spec.StepConfig(temperature=2.0, seed=11)
    for s in range(n):
        r = spec.speculative_step(tm.draft_next, tm.target_rows, [0], 1, s, 0, cfg, 0)
        cnt[r.emitted[0]] += 1
    want = np.sqrt(p) / np.sqrt(p).sum()
    assert np.max(np.abs(cnt / n - want)) < 4 * 0.5 / math.sqrt(n)


def test_forced_mode_mean_accept_matches_closed_form():
    # i.i.d. acceptance alpha: E[A] = alpha (1 - alpha^gamma) / (1 - alpha) (exact form of the
    # "about gamma*alpha + 1 tokens per step" estimate of the Background section)
    tm = _Tables([[0.25] * 4] * 4, [[0.25] * 4] * 4)
    for alpha, gamma in ((0.3, 4), (0.6, 2), (0.9, 8)):
        cfg = spec.StepConfig(temperature=1.0, seed=3, accept_mode=spec.FORCED_MODE, alpha=[alpha])
        n, g0, tot, sq = 6000, 0, 0, 0
        seen = set()
        for s in range(n):
            r = spec.speculative_step(tm.draft_next, tm.target_rows, [0], gamma, s, 0, cfg, g0)
            tot += r.accepted
            sq += r.accepted**2
            g0 += len(r.emitted)
        mean = tot / n
        want = alpha * (1 - alpha**gamma) / (1 - alpha)
        sd = math.sqrt(max(sq / n - mean**2, 1e-12) / n)
        assert abs(mean - want) < 4 * sd + 1e-3


def test_forced_landscape_is_shared_by_all_controllers():
    # the forced draw of generated index g does not depend on the step that reaches it
    seed = 9
    for g in (0, 1, 17):
        a = philox.forced_uniform(seed, g, 0)
        assert a == philox.uniform(seed, g, 0, philox.FORCED, 0)
    tm = _Tables([[0.25] * 4] * 4, [[0.25] * 4] * 4)
    alpha = [0.9] * 32 + [0.3] * 32
    cfg = spec.StepConfig(temperature=1.0, seed=seed, accept_mode=spec.FORCED_MODE, alpha=alpha)
    # per-token acceptance bits along the generated sequence, for two different controllers
    def accepted_bits(ctrl):
        res = spec.generate(tm.draft_next, tm.target_rows, [0], 48, ctrl, cfg)
        bits, g = {}, 0
        for st in res.steps:
            for i in range(st.k):
                if i < st.accepted:
                    bits[g + i] = 1
                elif i == st.accepted:
                    bits[g + i] = 0
            g += len(st.emitted)
        return bits
    b1 = accepted_bits(gt.FixedGamma(3))
    b2 = accepted_bits(gt.Controller(gt.Params(gamma_max=8), 4))
    common = set(b1) & set(b2)
    assert len(common) > 10
    assert all(b1[g] == b2[g] for g in common)


def test_early_stop_keeps_the_low_confidence_token():
    # draft law puts 0.4 on its top token; tau = 0.5 stops after the first draft token
    q = np.array([0.4, 0.3, 0.2, 0.1])
    tm = _Tables([q] * 4, [q] * 4)
    cfg = spec.StepConfig(temperature=1.0, seed=1, tau=0.5)
    r = spec.speculative_step(tm.draft_next, tm.target_rows, [0], 5, 0, 0, cfg, 0)
    assert r.k == 1 and len(r.drafted) == 1 and r.accepted == 1  # p == q: accepted
    assert len(r.emitted) == 2
    cfg2 = spec.StepConfig(temperature=1.0, seed=1, tau=0.35)
    r2 = spec.speculative_step(tm.draft_next, tm.target_rows, [0], 5, 0, 0, cfg2, 0)
    assert r2.k == 5
    # greedy: confidence is measured at T_eff = 1
    cfg3 = spec.StepConfig(temperature=0.0, tau=0.5)
    r3 = spec.speculative_step(tm.draft_next, tm.target_rows, [0], 5, 0, 0, cfg3, 0)
    assert r3.k == 1 and r3.conf[0] == pytest.approx(0.4)


# ---- margins: how far a decision is from flipping (the parity tests compare integers only where the
# margin exceeds the measured float error, so a margin that came out too large would hide a real
# disagreement and one that came out too small would excuse it) --------------------------------------

def test_top2_gap_hand_values():
    assert S.top2_gap(np.array([1.0, 3.5, 2.0, 3.0])) == 0.5
    assert S.top2_gap(np.array([-4.0, -1.5, -9.0])) == 2.5
    assert S.top2_gap(np.array([2.0, 7.0, 7.0, 1.0])) == 0.0       # tie at the top
    assert S.top2_gap(np.array([5.0, -5.0])) == 10.0
    assert S.top2_gap(np.array([3.0])) == float("inf")              # nothing to overtake
    # brute force: the gap is the smallest raise of a non-top entry that changes (or ties) the argmax
    rng = np.random.default_rng(0)
    for _ in range(50):
        x = rng.normal(size=7)
        top = int(np.argmax(x))
        want = min(x[top] - x[j] for j in range(7) if j != top)
        assert S.top2_gap(x) == pytest.approx(want, abs=0)


def test_inverse_cdf_margin_hand_values():
    # weights (1, 2, 1): W = 4, edges of the CDF at 1, 3, 4; every number below is dyadic, so exact
    w = np.array([1.0, 2.0, 1.0])
    assert S.inverse_cdf(w, 0.5) == (1, 0.25)        # u W = 2: 1 above the edge at 1, 1 below the edge at 3
    assert S.inverse_cdf(w, 0.125) == (0, 0.125)     # u W = 0.5: first cell, only its upper edge counts
    assert S.inverse_cdf(w, 0.8125) == (2, 0.0625)   # u W = 3.25: 0.25 above the edge at 3
    assert S.inverse_cdf(w, 0.25) == (1, 0.0)        # exactly on an edge: c_0 > u W fails, next cell, no margin
    assert S.inverse_cdf(w, 0.3125) == (1, 0.0625)   # u W = 1.25
    # unnormalised weights give the same answers
    assert S.inverse_cdf(8.0 * w, 0.8125) == (2, 0.0625)


def test_inverse_cdf_margin_is_the_distance_to_a_different_draw():
    rng = np.random.default_rng(1)
    for _ in range(200):
        V = int(rng.integers(2, 9))
        w = rng.dirichlet(np.ones(V))
        u = float(rng.random())
        j, m = S.inverse_cdf(w, u)
        assert m >= 0.0
        # moving u by less than the margin keeps the draw
        for d in (-0.98 * m, 0.98 * m):
            if 0.0 <= u + d < 1.0:
                assert S.inverse_cdf(w, u + d)[0] == j
        # moving it by a little more, towards the nearer edge, changes it (unless that runs off [0, 1))
        c = np.cumsum(w)
        lo = c[j - 1] if j > 0 else 0.0
        down_nearer = j > 0 and (u - lo) <= (c[j] - u)
        d = -(m + 1e-9) if down_nearer else (m + 1e-9)
        if 0.0 <= u + d < 1.0 and (down_nearer or j < V - 1):
            assert S.inverse_cdf(w, u + d)[0] != j


def test_accept_margin_hand_values():
    # u q < p; margin |u q - p| / max(p, q); dyadic numbers, exact
    assert S.accept_test(0.25, 0.5, 0.25) == (True, 0.25)    # 0.125 < 0.25, distance 0.125 over 0.5
    assert S.accept_test(0.25, 0.5, 0.75) == (False, 0.25)   # 0.375 >= 0.25
    assert S.accept_test(0.5, 0.25, 0.5) == (True, 0.75)     # p > q: 0.125 against 0.5
    assert S.accept_test(0.25, 0.5, 0.5) == (False, 0.0)     # u q == p: refused (strict test), no margin
    assert S.accept_test(0.0, 0.5, 0.0) == (False, 0.0)


def test_accept_margin_bounds_the_relative_change_that_flips():
    rng = np.random.default_rng(2)
    for _ in range(300):
        p, q, u = float(rng.random()), float(rng.random()), float(rng.random())
        ok, m = S.accept_test(p, q, u)
        # a relative change of p or q below the margin cannot flip the decision
        for f in (1 - 0.98 * m, 1 + 0.98 * m):
            assert S.accept_test(p * f, q, u)[0] == ok
            assert S.accept_test(p, q * f, u)[0] == ok
        # where p is the larger of the two, the margin is exactly the relative drop of p that flips it
        if p >= q and m < 1.0:
            assert S.accept_test(p * (1 - m - 1e-9), q, u)[0] is False


# ---- the synthetic confidence of forced mode -------------------------------------------------------

def _fixed_uniform(values, log):
    def u(s, i, purpose, b):
        log.append((s, i, purpose, b))
        return values[(s, i, purpose, b)] if (s, i, purpose, b) in values else 0.75
    return u


def test_forced_confidence_hand_values():
    # conf_i = clamp(alpha(g) + (0.5 - u(g, 0, FORCED, b)) / 2, 0, 1) with g = g0 + i - 1: the same draw that decides
    # the acceptance of position g, so the confidence is high exactly where acceptance is likely
    tm = _Tables([[0.25] * 4] * 4, [[0.25] * 4] * 4)
    b, g0 = 3, 10
    vals = {(10, 0, philox.FORCED, b): 0.25,      # 0.5 + 0.125        = 0.625
            (11, 0, philox.FORCED, b): 0.0,       # 0.875 + 0.25       = 1.125 -> 1
            (12, 0, philox.FORCED, b): 0.875,     # 0.125 - 0.1875     < 0     -> 0
            (13, 0, philox.FORCED, b): 0.5}       # 0.375 + 0          = 0.375
    alpha = [0.0] * 10 + [0.5, 0.875, 0.125, 0.375]
    log = []
    cfg = spec.StepConfig(temperature=1.0, accept_mode=spec.FORCED_MODE, alpha=alpha, tau=0.0)
    r = spec.speculative_step(tm.draft_next, tm.target_rows, [0], 4, 7, b, cfg, g0, uniform=_fixed_uniform(vals, log))
    assert r.conf == [0.625, 1.0, 0.0, 0.375]
    # the confidence of row i reads the counter of generated index g0 + i - 1, row 0, purpose FORCED
    forced_reads = [c for c in log if c[2] == philox.FORCED]
    assert set(forced_reads) == set(vals)
    # acceptance of the same positions: u < alpha -> 0.25 < 0.5 yes, 0 < 0.875 yes, 0.875 < 0.125 no
    assert r.accepted == 2
    # GammaTune+ threshold on that signal: tau = 0.7 stops at the first row (0.625 < 0.7), the token is kept
    cfg_t = spec.StepConfig(temperature=1.0, accept_mode=spec.FORCED_MODE, alpha=alpha, tau=0.7)
    r2 = spec.speculative_step(tm.draft_next, tm.target_rows, [0], 4, 7, b, cfg_t, g0, uniform=_fixed_uniform(vals, []))
    assert r2.k == 1 and r2.conf == [0.625] and r2.accepted == 1
    # tau = 0.5: rows 1 and 2 pass (0.625, 1.0), row 3 stops (0.0)
    cfg_u = spec.StepConfig(temperature=1.0, accept_mode=spec.FORCED_MODE, alpha=alpha, tau=0.5)
    r3 = spec.speculative_step(tm.draft_next, tm.target_rows, [0], 4, 7, b, cfg_u, g0, uniform=_fixed_uniform(vals, []))
    assert r3.k == 3 and r3.accepted == 2
    stops = [(d.row, d.value) for d in r3.decisions if d.kind == "stop"]
    assert stops == [(1, 0), (2, 0), (3, 1)]
    # margins of the stop decisions: |conf - tau| / tau
    m = [d.margin for d in r3.decisions if d.kind == "stop"]
    assert m == [0.25, 1.0, 1.0]


def test_forced_confidence_with_the_real_generator():
    # one alpha, one Philox counter: the uniform is the known generator's word 0 >> 8 over 2^24
    seed, g, b = 5, 2, 1
    w0 = philox.philox4x32_10((g, 0, philox.FORCED, b), philox.seed_key(seed))[0]
    u = (w0 >> 8) / 2.0**24
    tm = _Tables([[0.25] * 4] * 4, [[0.25] * 4] * 4)
    cfg = spec.StepConfig(temperature=1.0, seed=seed, accept_mode=spec.FORCED_MODE, alpha=[0.5])
    r = spec.speculative_step(tm.draft_next, tm.target_rows, [0], 1, 0, b, cfg, g)
    assert r.conf == [min(1.0, max(0.0, 0.5 + (0.5 - u) * 0.5))]
    assert r.accepted == int(u < 0.5)
