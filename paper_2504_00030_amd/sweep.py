"""Controllers under the same forced acceptance landscapes, on the 8B-shaped pair (synthetic stand-in for the
paper's comparison across initial speculation lengths; Experimental Details section, initial gamma in
{1..8, 12, 16, 20, 24}).

    python -m paper_2504_00030_amd.sweep [--pair 8b] [--n-generate 256] [--prompt-len 256]

For every landscape (alpha constant 0.3 / 0.6 / 0.9, and alternating 0.9 / 0.3 every 32 tokens) it times one
generation per initial gamma with: fixed gamma; fixed gamma with the confidence stop alone (early stop, no
controller); GammaTune; GammaTune+ (controller and confidence stop).  Prints one line per run and a table of
mean +- std tokens/s across the initial gammas.  All controllers meet the same landscape: the forced accept
bits and the synthetic confidence are functions of the generated-token index.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

GAMMAS = [1, 2, 3, 4, 5, 6, 7, 8, 12, 16, 20, 24]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--pair", default="8b")
    ap.add_argument("--n-generate", type=int, default=256)
    ap.add_argument("--prompt-len", type=int, default=256)
    ap.add_argument("--temperature", type=float, default=0.7)
    ap.add_argument("--out", default="")
    args = ap.parse_args()
    import torch
    import synth
    import paper_2504_00030_amd as pk

    cfg = synth.pair(args.pair)
    Wt, Wd = synth.make_pair_weights(cfg, 0, device="cuda")
    torch.cuda.synchronize()
    gmax = max(GAMMAS)
    prompts = synth.make_prompts(1, args.prompt_len, cfg.target.vocab, 7)
    tau = float(np.float32(0.4))
    eng = pk.SpecEngine(cfg.target, Wt, cfg.draft, Wd, batch=1, max_seq=args.prompt_len + args.n_generate + 2 * gmax + 8,
                        gamma_max=gmax, temperature=args.temperature, seed=0, accept_mode=pk.ACCEPT_FORCED, use_graphs=True)
    landscapes = {"alpha 0.3": synth.alpha_constant(0.3, 4), "alpha 0.6": synth.alpha_constant(0.6, 4),
                  "alpha 0.9": synth.alpha_constant(0.9, 4),
                  "alpha 0.9/0.3 every 32": synth.alpha_piecewise(args.n_generate + 2 * gmax + 8, 32)}
    methods = ["fixed", "fixed + confidence stop", "GammaTune", "GammaTune+"]
    rows = []
    for lname, alpha in landscapes.items():
        eng.set_forced_alpha(alpha)
        for method in methods:
            eng.set_early_stop(tau if method in ("fixed + confidence stop", "GammaTune+") else 0.0)
            for g0 in GAMMAS:
                rates = []
                for rep in range(2):  # the first repetition also captures the graphs this run needs
                    ctrl = (pk.FixedGamma(g0) if method.startswith("fixed")
                            else pk.GammaTune(eta=0.25, delta=1, gamma_min=1, gamma_max=gmax, gamma0=g0))
                    eng.prefill(prompts)
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    gen = steps = acc = 0
                    while gen < args.n_generate:
                        g = ctrl.gamma
                        eng.draft(g)
                        eng.verify(g)
                        A, y, k = eng.accept()
                        ctrl.update(int(A[0]), int(k[0]))
                        gen += int(A[0]) + 1
                        acc += int(A[0])
                        steps += 1
                    torch.cuda.synchronize()
                    rates.append(args.n_generate / (time.perf_counter() - t0))
                rows.append(dict(landscape=lname, method=method, gamma0=g0, tokens_per_s=rates[-1], steps=steps,
                                 tokens_per_step=gen / steps))
                print(f"{lname:24s} {method:24s} gamma0 {g0:2d}: {rates[-1]:7.1f} tokens/s, {gen / steps:5.2f} tokens/step",
                      flush=True)
    eng.close()
    print()
    print("| landscape | " + " | ".join(methods) + " |")
    print("|---|" + "---|" * len(methods))
    for lname in landscapes:
        cells = []
        for method in methods:
            v = np.array([r["tokens_per_s"] for r in rows if r["landscape"] == lname and r["method"] == method])
            best = GAMMAS[int(v.argmax())]
            cells.append(f"{v.mean():.0f} ± {v.std():.0f} (best {v.max():.0f} at {best})")
        print(f"| {lname} | " + " | ".join(cells) + " |")
    if args.out:
        with open(args.out, "w") as f:
            json.dump(rows, f)


if __name__ == "__main__":
    main()
