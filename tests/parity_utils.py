"""Shared helpers of the GPU parity tests.

The HIP library and the CPU oracle are driven in lock-step on the same seeded inputs.  After every
speculative step the library's integers (drafted tokens, drafted count, accepted count, emitted
token, next gamma) and logits are compared with the oracle's.  A decision may differ only where the
oracle reports a margin below the float error measured on that step's logits, and the library's token
must then still lie within that error of the oracle's draw; in that case the step is counted as
"skipped", and the library is restarted from the ORACLE's token sequence (spec_prefill_ragged +
spec_debug_set_step), so that later steps are compared on identical prefixes again.  Nothing the
library computes ever flows into the oracle.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np

import synth
from oracle import gammatune as ogt
from oracle import model as om
from oracle import philox as ophilox
from oracle import sampling as osamp
from oracle import spec as ospec

# max-abs logit error relative to max |logit|; 8-bit weights are exact in the kernels (int8 -> bf16), so the
# activations' two bf16 terms bound the error as for bf16 weights
TOL = {"fp32": 1e-4, "bf16": 1e-2, "q8": 1e-2}


def oshape(ms: synth.ModelShape) -> om.Shape:
    return om.Shape(ms.n_layers, ms.d_model, ms.n_q_heads, ms.n_kv_heads, ms.head_dim, ms.d_ffn, ms.vocab,
                    ms.rope_theta, ms.rms_eps, ms.dtype in ("bf16", "q8"))


def to_gpu(W):
    return {k: ([t.cuda().contiguous() for t in v] if isinstance(v, list) else v.cuda().contiguous()) for k, v in W.items()}


@dataclass
class Compare:
    steps_total: int = 0          # (sequence, step) pairs compared
    steps_clean: int = 0          # ... with every decision identical
    resyncs: int = 0
    decisions_compared: int = 0
    decisions_skipped: int = 0    # differed below the margin threshold
    max_logit_err: float = 0.0    # relative to max |logit|
    kappa_prob_max: float = 0.0   # largest probability threshold any step used (8 x measured logit error / T)
    failures: List[str] = field(default_factory=list)
    skipped: List[str] = field(default_factory=list)
    trace: List[dict] = field(default_factory=list)

    @property
    def coverage(self) -> float:
        return self.steps_clean / max(1, self.steps_total)


class ScriptGamma:
    """Speculation lengths read from a list, one per step, repeating (test driver only: no rule of the method)."""

    def __init__(self, script):
        self.script, self.i = list(script), 0

    @property
    def gamma(self):
        return self.script[self.i % len(self.script)]

    def update(self, accepted, drafted):
        self.i += 1
        return self.gamma


def make_controllers(kind: str, n: int, gamma_max: int, which: str):
    """kind: 'fixed<g>', 'spread' (sequence b keeps the fixed gamma 1 + 3 b mod gamma_max: every step's sequences
    differ in their rows), 'script:g1,g2,...' (every sequence walks the same list) or 'gammatune'; which: 'gpu'
    (C controller) or 'oracle'."""
    import paper_2504_00030_amd as pk
    out = []
    for b in range(n):
        if kind.startswith("script:"):
            out.append(ScriptGamma(int(g) for g in kind[7:].split(",")))
        elif kind == "spread":
            g = 1 + (3 * b) % gamma_max
            out.append(pk.FixedGamma(g) if which == "gpu" else ogt.FixedGamma(g))
        elif kind.startswith("fixed"):
            g = int(kind[5:])
            out.append(pk.FixedGamma(g) if which == "gpu" else ogt.FixedGamma(g))
        elif which == "gpu":
            out.append(pk.GammaTune(eta=0.25, delta=1, gamma_min=1, gamma_max=gamma_max, gamma0=4))
        else:
            out.append(ogt.Controller(ogt.Params(0.25, 1, 1, gamma_max), 4))
    return out


def _cdf_distance(w, u: float, tok: int) -> float:
    """How far u W lies from the CDF cell of token `tok` under weights w, over W (0 when inside the cell)."""
    c = np.cumsum(np.asarray(w, dtype=np.float64))
    W = float(c[-1])
    if not (W > 0.0) or tok < 0 or tok >= c.shape[0]:
        return float("inf")
    t = u * W
    lo = float(c[tok - 1]) if tok > 0 else 0.0
    hi = float(c[tok])
    if lo <= t < hi:
        return 0.0
    return min(abs(t - lo), abs(t - hi)) / W


def _compare_step(res: Compare, tag: str, r, gamma: int, gk: int, gA: int, gy: int, gdrafted, ql, pl, dtype: str,
                  temperature: float, *, s: int, b: int, seed: int, forced: bool) -> bool:
    """Compare one sequence's step; returns True when every decision matched.

    Thresholds come from the float error MEASURED on this step's logits, eps = max |gpu - oracle| over the rows
    whose inputs agree (at least 1 % of the tolerance budget): a logit gap survives while it exceeds 2 eps, a
    relative probability or CDF position moves by at most 4 eps / T, so decisions are demanded equal where the
    oracle's margin exceeds kappa_logit = 4 eps resp. kappa_prob = 8 eps / T (the residual draw divides by its
    total mass W_res = sum max(0, p - q), which the same perturbation is measured against).  A decision that
    differs below its threshold is still checked for validity: the library's token must lie within the threshold
    of the oracle's own draw (CDF distance of u, or logit distance from the top).  In forced-acceptance mode the
    stop signal and the accept bits do not depend on the tokens, so (k, A) must agree on every step."""
    scale = max(float(np.abs(r.p_logits).max()), float(np.abs(np.stack(r.q_logits)).max()))
    if not (np.isfinite(ql[: max(gk, 1)]).all() and np.isfinite(pl[: gk + 1]).all()):
        res.failures.append(f"{tag}: non-finite logits from the library")
        return False
    T = temperature if temperature > 0 else 1.0
    # logits of rows whose inputs (the drafted tokens before them) agree
    n_agree = 0
    while n_agree < min(r.k, gk) and gdrafted[n_agree] == r.drafted[n_agree]:
        n_agree += 1
    errs = []
    for i in range(min(r.k, gk, n_agree + 1)):
        e_abs = float(np.abs(ql[i] - r.q_logits[i]).max())
        errs.append(e_abs)
        if not e_abs / scale <= TOL[dtype]:
            res.failures.append(f"{tag}: draft logits row {i} err {e_abs / scale:.3e}")
    for i in range(min(r.k, gk, n_agree) + 1):
        e_abs = float(np.abs(pl[i] - r.p_logits[i]).max())
        errs.append(e_abs)
        if not e_abs / scale <= TOL[dtype]:
            res.failures.append(f"{tag}: target logits row {i} err {e_abs / scale:.3e}")
    res.max_logit_err = max(res.max_logit_err, max(errs, default=0.0) / scale)
    eps = max(max(errs, default=0.0), 1e-2 * TOL[dtype] * scale)
    k_logit = 4.0 * eps
    k_prob = 8.0 * eps / T
    res.kappa_prob_max = max(res.kappa_prob_max, k_prob)

    def uniform(i, purpose):
        return ophilox.uniform(seed, s, i, purpose, b)

    def token_is_valid(dcs, got, kappa) -> bool:
        """The library's token against the oracle's own distribution and uniform."""
        if got is None:
            return False
        if dcs.kind == "draft":
            row, purpose, lq = dcs.row, ophilox.DRAFT, r.q_logits[dcs.row - 1]
            if dcs.scale == "logit":
                return float(lq.max() - lq[got]) <= kappa
            return _cdf_distance(osamp.softmax_T(lq, T), uniform(row, purpose), got) <= kappa
        lp = r.p_logits[dcs.row - 1]
        if dcs.scale == "logit":
            return float(lp.max() - lp[got]) <= kappa
        if dcs.kind == "bonus":
            return _cdf_distance(osamp.softmax_T(lp, T), uniform(dcs.row, ophilox.BONUS), got) <= kappa
        w = osamp.residual_weights(osamp.softmax_T(lp, T), osamp.softmax_T(r.q_logits[dcs.row - 1], T))
        if not (w.sum() > 0.0):
            w = osamp.softmax_T(lp, T)
        return _cdf_distance(w, uniform(dcs.row, ophilox.RESID), got) <= kappa

    diverged = False
    for dcs in r.decisions:
        kappa = k_logit if dcs.scale == "logit" else k_prob
        if dcs.kind == "resid" and dcs.scale == "prob":
            w_res = float(osamp.residual_weights(osamp.softmax_T(r.p_logits[dcs.row - 1], T),
                                                 osamp.softmax_T(r.q_logits[dcs.row - 1], T)).sum())
            if w_res > 0.0:
                kappa = k_prob / w_res
        if diverged:
            # only what does not depend on the tokens is still comparable: forced-mode stop and accept bits
            if not (forced and dcs.kind in ("stop", "accept")):
                continue
        if dcs.kind == "draft":
            got = gdrafted[dcs.row - 1] if dcs.row - 1 < len(gdrafted) else None
        elif dcs.kind == "stop":
            if dcs.row < gk:
                got = 0
            elif dcs.row == gk:
                got = 1 if gk < gamma else dcs.value  # reaching gamma ends drafting either way
            else:
                got = None
        elif dcs.kind == "accept":
            got = int(gA >= dcs.row)
        else:  # resid / bonus
            got = gy
        res.decisions_compared += 1
        if got is None or got != dcs.value:
            is_token = dcs.kind in ("draft", "resid", "bonus")
            if dcs.margin > kappa:
                res.failures.append(f"{tag}: {dcs.kind} row {dcs.row}: gpu {got} != oracle {dcs.value} "
                                    f"(margin {dcs.margin:.3e} > {kappa:.3e})")
                return False
            if is_token and not token_is_valid(dcs, got, kappa):
                res.failures.append(f"{tag}: {dcs.kind} row {dcs.row}: gpu token {got} lies further than {kappa:.3e} "
                                    f"from the oracle's draw {dcs.value}")
                return False
            res.decisions_skipped += 1
            res.skipped.append(f"{tag}: {dcs.kind} row {dcs.row} margin {dcs.margin:.3e}")
            if forced and is_token:
                diverged = True
                continue
            return False
    if diverged:
        if (gk, gA) != (r.k, r.accepted):
            res.failures.append(f"{tag}: forced mode (k,A) gpu {(gk, gA)} != oracle {(r.k, r.accepted)}")
        return False
    if (gk, gA, gy) != (r.k, r.accepted, r.y):
        res.failures.append(f"{tag}: (k,A,y) gpu {(gk, gA, gy)} != oracle {(r.k, r.accepted, r.y)}")
        return False
    return True


def run_lockstep(eng, cfg: synth.PairConfig, Wt_np, Wd_np, prompts, n_generate, *, controller: str,
                 temperature: float, seed: int, accept_mode: int = 0, alpha=None, tau: float = 0.0,
                 max_failures: int = 5) -> Compare:
    dtype = cfg.target.dtype
    res = Compare()
    forced = accept_mode == 1
    B = prompts.shape[0]
    n0 = prompts.shape[1]
    pairs = [ospec.TransformerPair(oshape(cfg.target), Wt_np, oshape(cfg.draft), Wd_np) for _ in range(B)]
    octl = make_controllers(controller, B, cfg.gamma_max, "oracle")
    gctl = make_controllers(controller, B, cfg.gamma_max, "gpu")
    scfg = ospec.StepConfig(temperature=temperature, seed=seed, accept_mode=accept_mode, tau=tau,
                            alpha=None if alpha is None else [float(a) for a in alpha])
    toks = [[int(t) for t in prompts[b]] for b in range(B)]
    eng.prefill(prompts)
    s = 0
    while min(len(t) for t in toks) - n0 < n_generate and len(res.failures) < max_failures:
        gammas = np.array([c.gamma for c in octl], dtype=np.int32)
        ggam = [c.gamma for c in gctl]
        if ggam != gammas.tolist():
            res.failures.append(f"step {s}: gamma gpu {ggam} != oracle {gammas.tolist()}")
            break
        eng.draft(gammas if B > 1 else int(gammas[0]))
        eng.verify(int(gammas.max()))
        q = eng.debug_logits(0)
        drafted = [eng.debug_drafted(b) for b in range(B)]
        A, y, k = eng.accept()
        p = eng.debug_logits(1)
        res.trace.append({"gamma": gammas.copy(), "A": A.copy(), "y": y.copy(), "k": k.copy()})
        resync = False
        for b in range(B):
            r = ospec.speculative_step(pairs[b].draft_next, pairs[b].target_rows, toks[b], int(gammas[b]), s, b, scfg,
                                       len(toks[b]) - n0, keep_logits=True)
            res.steps_total += 1
            ok = _compare_step(res, f"seq {b} step {s}", r, int(gammas[b]), int(k[b]), int(A[b]), int(y[b]), drafted[b],
                               q[b], p[b], dtype, temperature, s=s, b=b, seed=seed, forced=forced)
            toks[b].extend(r.emitted)
            octl[b].update(r.accepted, r.k)
            if ok or forced:
                # forced mode: the library's own (A, k) drive its controller on every step, clean or not, and the
                # check at the top of the loop demands the same next gamma as the oracle's
                gctl[b].update(int(A[b]), int(k[b]))
            if ok:
                res.steps_clean += 1
            else:
                resync = True
        s += 1
        if resync:
            # restart the library from the oracle's sequences and controller states
            res.resyncs += 1
            eng.prefill_ragged(toks)
            eng.set_step(s, [n0] * B)
            for b in range(B):
                if hasattr(gctl[b], "state") and not forced:
                    gctl[b].state.gamma_bar = octl[b].gamma_bar
                    gctl[b].state.gamma = octl[b].gamma
    if not res.failures:
        for b in range(B):
            got = eng.read_tokens(b).tolist()
            if got != toks[b]:
                res.failures.append(f"seq {b}: final tokens differ")
    res.tokens = [t[: n0 + n_generate] for t in toks]
    return res
