"""One speculative-decoding step and the generation loop around it.

Test infrastructure only (see oracle/__init__.py).

Follows the Background section: the draft model samples gamma tokens
autoregressively, the target model scores all of them in one pass, and the
accepted prefix plus one target-distributed token is emitted, so that the
output is distributed as target-only sampling.  The GammaTune section supplies
gamma for the next step from A (oracle.gammatune); GammaTune+ additionally
stops drafting when the draft's top probability falls below tau.

Step, for a prefix t[0..n) and planned length gamma (s = step ordinal,
b = sequence index, g0 = tokens generated before the step):

  for i = 1..gamma
      lq_i = draft logits for the token after  t + x_1..x_{i-1}
      x_i  = argmax lq_i                      (T == 0)
           = inverse-CDF draw from softmax(lq_i / T) with u(s, i, DRAFT, b)
      conf_i = max softmax(lq_i / T_eff), T_eff = T if T > 0 else 1
               (forced mode: conf_i = clamp(alpha(g) + (0.5 - u(g, FORCED)) / 2, 0, 1) with
                g = g0+i-1, a synthetic confidence centred on the acceptance rate of the
                position and monotone in the hidden acceptance draw)
      if tau > 0 and conf_i < tau: stop drafting, x_i is kept        [k = i]
  k = number of drafted tokens
  lp_1..lp_{k+1} = target logits for the tokens after t, t+x_1, ..., t+x_1..x_k
  A = number of leading i in 1..k that pass
        natural : u(s, i, ACCEPT, b) * q_i(x_i) < p_i(x_i)
        greedy  : x_i == argmax lp_i
        forced  : u(g0+i-1, FORCED) < alpha(g0+i-1)
  y = A < k : greedy -> argmax lp_{A+1}
              else   -> draw from norm(max(0, p_{A+1} - q_{A+1})) with u(s, A+1, RESID, b)
      A == k: greedy -> argmax lp_{k+1}
              else   -> draw from p_{k+1} with u(s, k+1, BONUS, b)
  emit x_1..x_A, y

The models enter only through two callables, so table-driven toy models can
be plugged in for the brute-force distribution checks.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Optional, Sequence

import numpy as np

from . import philox
from . import sampling as S
from .model import KVCache, Shape, forward

NATURAL, FORCED_MODE = 0, 1


@dataclass
class StepConfig:
    temperature: float = 0.0
    seed: int = 0
    accept_mode: int = NATURAL
    tau: float = 0.0
    alpha: Optional[Sequence[float]] = None  # forced mode: alpha per generated index (last value repeats)


@dataclass
class Decision:
    kind: str        # "draft", "accept", "resid", "bonus", "stop"
    row: int         # i, 1-based
    value: int       # token id, or 0/1 for accept and stop
    margin: float    # distance from flipping (logit gap for greedy / argmax kinds)
    scale: str       # "logit" (margin is a logit gap), "prob" (relative probability / CDF distance)


@dataclass
class StepResult:
    gamma: int
    drafted: List[int]
    k: int
    accepted: int
    y: int
    emitted: List[int]
    decisions: List[Decision] = field(default_factory=list)
    conf: List[float] = field(default_factory=list)
    q_logits: List[np.ndarray] = field(default_factory=list)
    p_logits: Optional[np.ndarray] = None


def _alpha_at(alpha: Sequence[float], g: int) -> float:
    return float(alpha[g]) if g < len(alpha) else float(alpha[-1])


def speculative_step(
    draft_next: Callable[[List[int]], np.ndarray],
    target_rows: Callable[[List[int], int], np.ndarray],
    prefix: List[int],
    gamma: int,
    s: int,
    b: int,
    cfg: StepConfig,
    g0: int,
    uniform: Optional[Callable[[int, int, int, int], float]] = None,
    keep_logits: bool = False,
) -> StepResult:
    """draft_next(tokens) -> logits [V] of the next token; target_rows(tokens, k)
    -> logits [k+1, V] of the tokens following tokens[:len-k], ..., tokens[:len]."""
    if uniform is None:
        uniform = lambda s_, i_, purpose_, b_: philox.uniform(cfg.seed, s_, i_, purpose_, b_)
    T = float(cfg.temperature)
    greedy = T == 0.0
    T_eff = T if T > 0.0 else 1.0
    forced = cfg.accept_mode == FORCED_MODE
    res = StepResult(gamma=gamma, drafted=[], k=0, accepted=0, y=-1, emitted=[])

    cur = list(prefix)
    q_rows: List[np.ndarray] = []
    for i in range(1, gamma + 1):
        lq = np.asarray(draft_next(cur), dtype=np.float64)
        q_rows.append(lq)
        if greedy:
            x = S.argmax_lowest(lq)
            res.decisions.append(Decision("draft", i, x, S.top2_gap(lq), "logit"))
        else:
            x, mg = S.inverse_cdf(S.softmax_T(lq, T), uniform(s, i, philox.DRAFT, b))
            res.decisions.append(Decision("draft", i, x, mg, "prob"))
        res.drafted.append(x)
        cur.append(x)
        if forced:
            g = g0 + i - 1
            conf = _alpha_at(cfg.alpha, g) + (0.5 - uniform(g, 0, philox.FORCED, b)) * 0.5
            conf = min(1.0, max(0.0, conf))
        else:
            conf = S.top_probability(lq, T_eff)
        res.conf.append(conf)
        if cfg.tau > 0.0:
            stop = conf < cfg.tau
            rel = abs(conf - cfg.tau) / cfg.tau
            res.decisions.append(Decision("stop", i, int(stop), rel, "prob"))
            if stop:
                break
    k = len(res.drafted)
    res.k = k

    lp = np.asarray(target_rows(cur, k), dtype=np.float64)  # [k+1, V]
    assert lp.shape[0] == k + 1

    A = 0
    for i in range(1, k + 1):
        x = res.drafted[i - 1]
        if forced:
            u = uniform(g0 + i - 1, 0, philox.FORCED, b)
            ok = u < _alpha_at(cfg.alpha, g0 + i - 1)
            mg = float("inf")
            scale = "prob"
        elif greedy:
            top = S.argmax_lowest(lp[i - 1])
            ok = x == top
            # flips if another token overtakes the current argmax, or x overtakes it
            mg = S.top2_gap(lp[i - 1]) if ok else float(lp[i - 1][top] - lp[i - 1][x])
            scale = "logit"
        else:
            p_x = float(S.softmax_T(lp[i - 1], T)[x])
            q_x = float(S.softmax_T(q_rows[i - 1], T)[x])
            ok, mg = S.accept_test(p_x, q_x, uniform(s, i, philox.ACCEPT, b))
            scale = "prob"
        res.decisions.append(Decision("accept", i, int(ok), mg, scale))
        if not ok:
            break
        A += 1
    res.accepted = A

    if A < k:
        row = A + 1
        if greedy:
            y = S.argmax_lowest(lp[row - 1])
            res.decisions.append(Decision("resid", row, y, S.top2_gap(lp[row - 1]), "logit"))
        else:
            y, mg = S.sample_residual(
                S.softmax_T(lp[row - 1], T), S.softmax_T(q_rows[row - 1], T), uniform(s, row, philox.RESID, b)
            )
            res.decisions.append(Decision("resid", row, y, mg, "prob"))
    else:
        row = k + 1
        if greedy:
            y = S.argmax_lowest(lp[row - 1])
            res.decisions.append(Decision("bonus", row, y, S.top2_gap(lp[row - 1]), "logit"))
        else:
            y, mg = S.inverse_cdf(S.softmax_T(lp[row - 1], T), uniform(s, row, philox.BONUS, b))
            res.decisions.append(Decision("bonus", row, y, mg, "prob"))
    res.y = y
    res.emitted = res.drafted[:A] + [y]
    if keep_logits:
        res.q_logits = q_rows
        res.p_logits = lp
    return res


class TransformerPair:
    """Draft and target decoders with incremental caches behind the two callables."""

    def __init__(self, shape_t: Shape, W_t, shape_d: Shape, W_d):
        self.st, self.Wt, self.sd, self.Wd = shape_t, W_t, shape_d, W_d
        self._ct, self._tt = KVCache(shape_t), []
        self._cd, self._td = KVCache(shape_d), []

    @staticmethod
    def _sync(cache: KVCache, have: List[int], want: List[int], keep_back: int):
        """Truncate cache to the common prefix, leaving at least keep_back tokens to feed."""
        n = 0
        lim = min(len(have), len(want) - keep_back)
        while n < lim and have[n] == want[n]:
            n += 1
        cache.truncate(n)
        return n

    def draft_next(self, tokens: List[int]) -> np.ndarray:
        n = self._sync(self._cd, self._td, tokens, 1)
        out = forward(self.sd, self.Wd, tokens[n:], self._cd)
        self._td = list(tokens)
        return out[-1]

    def target_rows(self, tokens: List[int], k: int) -> np.ndarray:
        n = self._sync(self._ct, self._tt, tokens, k + 1)
        out = forward(self.st, self.Wt, tokens[n:], self._ct)
        self._tt = list(tokens)
        return out[-(k + 1):]


@dataclass
class GenerateResult:
    tokens: List[int]            # prompt + exactly n_generate tokens
    steps: List[StepResult]
    gammas: List[int]            # planned gamma of every step


def generate(
    draft_next,
    target_rows,
    prompt: Sequence[int],
    n_generate: int,
    controller,
    cfg: StepConfig,
    b: int = 0,
    keep_logits: bool = False,
    uniform=None,
) -> GenerateResult:
    """Run speculative steps until n_generate tokens exist; the surplus of the last step is dropped."""
    toks = list(int(t) for t in prompt)
    n0 = len(toks)
    steps: List[StepResult] = []
    gammas: List[int] = []
    s = 0
    while len(toks) - n0 < n_generate:
        gamma = int(controller.gamma)
        gammas.append(gamma)
        r = speculative_step(draft_next, target_rows, toks, gamma, s, b, cfg, len(toks) - n0, uniform, keep_logits)
        steps.append(r)
        toks.extend(r.emitted)
        controller.update(r.accepted, r.k)
        s += 1
    return GenerateResult(tokens=toks[: n0 + n_generate], steps=steps, gammas=gammas)


def target_only(target_rows, prompt: Sequence[int], n_generate: int, cfg: StepConfig, b: int = 0, uniform=None):
    """Plain autoregressive decoding with the target model (greedy, or one BONUS draw per token)."""
    if uniform is None:
        uniform = lambda s_, i_, purpose_, b_: philox.uniform(cfg.seed, s_, i_, purpose_, b_)
    toks = list(int(t) for t in prompt)
    for s in range(n_generate):
        lp = np.asarray(target_rows(toks, 0), dtype=np.float64)[-1]
        if cfg.temperature == 0.0:
            y = S.argmax_lowest(lp)
        else:
            y, _ = S.inverse_cdf(S.softmax_T(lp, cfg.temperature), uniform(s, 1, philox.BONUS, b))
        toks.append(y)
    return toks
