"""Shared helpers of the GPU parity tests: run the HIP library and the CPU oracle on the same seeded
inputs and compare them decision by decision."""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional

import numpy as np

import synth
from oracle import gammatune as ogt
from oracle import model as om
from oracle import spec as ospec

TOL = {"fp32": 1e-4, "bf16": 1e-2}  # max-abs logit error relative to max |logit|


def oshape(ms: synth.ModelShape) -> om.Shape:
    return om.Shape(ms.n_layers, ms.d_model, ms.n_q_heads, ms.n_kv_heads, ms.head_dim, ms.d_ffn, ms.vocab,
                    ms.rope_theta, ms.rms_eps, ms.dtype == "bf16")


def to_gpu(W):
    return {k: ([t.cuda().contiguous() for t in v] if isinstance(v, list) else v.cuda().contiguous()) for k, v in W.items()}


@dataclass
class Compare:
    steps_compared: int = 0
    steps_total: int = 0
    decisions_compared: int = 0
    diverged_at: Optional[str] = None      # description of the sub-margin decision that ended the comparison
    max_logit_err: float = 0.0             # relative to max |logit|
    failures: List[str] = None

    @property
    def coverage(self) -> float:
        return self.steps_compared / max(1, self.steps_total)


def make_controllers(kind: str, n: int, gamma_max: int, which: str):
    """kind: 'fixed<g>' or 'gammatune'; which: 'gpu' (C controller) or 'oracle'."""
    import paper_2504_00030_amd as pk
    out = []
    for _ in range(n):
        if kind.startswith("fixed"):
            g = int(kind[5:])
            out.append(pk.FixedGamma(g) if which == "gpu" else ogt.FixedGamma(g))
        else:
            if which == "gpu":
                out.append(pk.GammaTune(eta=0.25, delta=1, gamma_min=1, gamma_max=gamma_max, gamma0=4))
            else:
                out.append(ogt.Controller(ogt.Params(0.25, 1, 1, gamma_max), 4))
    return out


def compare_run(cfg: synth.PairConfig, Wt_np, Wd_np, prompts, n_generate, gpu_tokens, gpu_trace, *, controller: str,
                temperature: float, seed: int, accept_mode: int = 0, alpha=None, tau: float = 0.0) -> Compare:
    """Replay the run on the oracle, sequence by sequence, and compare with what the GPU produced."""
    dtype = cfg.target.dtype
    res = Compare(failures=[])
    B = prompts.shape[0]
    for b in range(B):
        pair = ospec.TransformerPair(oshape(cfg.target), Wt_np, oshape(cfg.draft), Wd_np)
        ctrl = make_controllers(controller, 1, cfg.gamma_max, "oracle")[0]
        scfg = ospec.StepConfig(temperature=temperature, seed=seed, accept_mode=accept_mode, tau=tau,
                                alpha=None if alpha is None else [float(a) for a in alpha])
        toks = [int(t) for t in prompts[b]]
        n0 = len(toks)
        s = 0
        alive = True
        res.steps_total += len(gpu_trace)
        for rec in gpu_trace:
            if not alive:
                break
            gamma = int(ctrl.gamma)
            if int(rec["gamma"][b]) != gamma:
                res.failures.append(f"seq {b} step {s}: gamma {int(rec['gamma'][b])} != oracle {gamma}")
                break
            gmax_step = int(rec["gamma"].max())
            r = ospec.speculative_step(pair.draft_next, pair.target_rows, toks, gamma, s, b, scfg, len(toks) - n0,
                                       keep_logits=True)
            scale = max(float(np.abs(r.p_logits).max()), float(np.abs(np.stack(r.q_logits)).max()))
            eps = TOL[dtype] * scale
            k_logit = 4.0 * eps
            k_prob = 8.0 * eps / (temperature if temperature > 0 else 1.0)
            gk, gA, gy = int(rec["k"][b]), int(rec["A"][b]), int(rec["y"][b])
            # logits of the rows both sides computed from the same prefix
            if "q_logits" in rec:
                ql = rec["q_logits"][b]
                gdrafted = rec.get("drafted")
                for i in range(min(r.k, gk)):
                    # row i is comparable when the drafted tokens before it agree
                    err = float(np.abs(ql[i] - r.q_logits[i]).max()) / scale
                    res.max_logit_err = max(res.max_logit_err, err)
                    if err > TOL[dtype]:
                        res.failures.append(f"seq {b} step {s}: draft logits row {i} err {err:.3e}")
                    if gdrafted is not None and int(gdrafted[b][i]) != r.drafted[i]:
                        break
            # decisions, in the oracle's order
            gpu_drafted = None if "drafted" not in rec else [int(t) for t in rec["drafted"][b][:gk]]
            ok_so_far = True
            for dcs in r.decisions:
                kappa = k_logit if dcs.scale == "logit" else k_prob
                if dcs.kind == "draft":
                    if gpu_drafted is None:
                        continue
                    got = gpu_drafted[dcs.row - 1] if dcs.row - 1 < len(gpu_drafted) else None
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
                    if dcs.margin > kappa:
                        res.failures.append(
                            f"seq {b} step {s}: {dcs.kind} row {dcs.row}: gpu {got} != oracle {dcs.value} "
                            f"(margin {dcs.margin:.3e} > {kappa:.3e})")
                    else:
                        res.diverged_at = f"seq {b} step {s} {dcs.kind} row {dcs.row} margin {dcs.margin:.3e}"
                    ok_so_far = False
                    break
            if not ok_so_far:
                alive = False
                break
            if "p_logits" in rec and gk == r.k and (gpu_drafted is None or gpu_drafted == r.drafted):
                pl = rec["p_logits"][b][: r.k + 1]
                err = float(np.abs(pl - r.p_logits).max()) / scale
                res.max_logit_err = max(res.max_logit_err, err)
                if err > TOL[dtype]:
                    res.failures.append(f"seq {b} step {s}: target logits err {err:.3e}")
            if (gk, gA, gy) != (r.k, r.accepted, r.y):
                res.failures.append(f"seq {b} step {s}: (k,A,y) gpu {(gk, gA, gy)} != oracle {(r.k, r.accepted, r.y)}")
                break
            toks.extend(r.emitted)
            ctrl.update(r.accepted, r.k)
            s += 1
            res.steps_compared += 1
        if alive and not res.failures:
            want = toks[: n0 + n_generate]
            got = [int(t) for t in gpu_tokens[b][: len(want)]]
            if got != want[: len(got)]:
                res.failures.append(f"seq {b}: final tokens differ")
    return res
