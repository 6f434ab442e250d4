#!/usr/bin/env python3
"""Speculative-decoding throughput on one MI355X.

A "step" is one whole generation over one batch of synthetic input: the prompt is prefilled
(untimed, reported separately) and then speculative steps (draft gamma tokens, verify gamma+1
rows, accept / resample, controller update) run until n_generate tokens exist.  The timed region
of a step is its decode loop, bracketed by device synchronisation on both sides.

Default workload: the 8B-shaped target with the 1B-shaped draft, batch 1, prompt 1024, 512 new
tokens, GammaTune+ (gamma in [1,16], tau 0.4), temperature 0.7, forced acceptance landscape that
alternates alpha = 0.9 / 0.3 every 32 tokens.  Weights are seeded random-init, generated on the GPU.

Prints ONE JSON line (see the keys below).  `roofline` times the dominant kernel (the target's
gate/up projection, which streams 2*d_ffn*d_model bf16 weights per launch) with HIP event pairs
around its launches on the engine's stream; `cpu_baseline` times the fp64 CPU oracle on a bounded
sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 matrix-core peak of the chip


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--pair", default="8b", choices=["tiny", "1b", "7b", "8b", "8b-q8", "13b"])
    ap.add_argument("--alpha", default="piecewise", help="piecewise | a constant such as 0.6")
    ap.add_argument("--controller", default="gammatune+", choices=["gammatune", "gammatune+", "fixed"])
    ap.add_argument("--gamma0", type=int, default=4)
    ap.add_argument("--temperature", type=float, default=0.7)
    ap.add_argument("--n-generate", type=int, default=0)
    ap.add_argument("--prompt-len", type=int, default=0)
    ap.add_argument("--no-graphs", action="store_true")
    ap.add_argument("--skip-cpu", action="store_true")
    ap.add_argument("--skip-roofline", action="store_true")
    ap.add_argument("--gemv-path", type=int, default=0)
    ap.add_argument("--attn-chunk", type=int, default=0)
    ap.add_argument("--host-loop", action="store_true", help="drive the steps from Python instead of spec_generate")
    ap.add_argument("--batch", type=int, default=1, help="sequences decoded in lock-step, one controller each "
                                                         "(the headline metric is batch 1)")
    ap.add_argument("--prefill-only", action="store_true",
                    help="time --steps prompt ingestions (after --warmup untimed ones) and print the prefill object alone")
    ap.add_argument("--accept", default="forced", choices=["forced", "natural"],
                    help="forced: seeded Bernoulli acceptance landscape (--alpha); natural: the accept test u q(x) < p(x)")
    ap.add_argument("--cpu-full", action="store_true",
                    help="CPU baseline: time two whole oracle steps at full depth instead of the 0-/1-layer extrapolation "
                         "(8B pair: about 75 GB of host memory and several minutes)")
    ap.add_argument("--verify-sweep", action="store_true",
                    help="verification-only sweep on the --pair's target (default there: 13b): rows x cache length x batch "
                         "on a seeded synthetic KV cache; prints one JSON object with a cell per combination")
    ap.add_argument("--sweep-rows", default="1,2,4,8,16")
    ap.add_argument("--sweep-kv", default="512,1024,2048,4096")
    ap.add_argument("--sweep-batch", default="1,4,8")
    ap.add_argument("--sweep-reps", type=int, default=20)
    ap.add_argument("--roofline-only", action="store_true",
                    help="skip the timed generations: prefill, the event-timed decode leg and the reference copy only "
                         "(a short run for profiler counter passes)")
    return ap.parse_args()


def decode_loop(eng, ctrls, n_generate):
    """Speculative steps until every sequence has n_generate new tokens; `ctrls`: one controller per sequence.
    Counts tokens up to n_generate per sequence.  The loop itself runs in the library (spec_generate)."""
    return eng.run(n_generate, ctrls)


def decode_loop_host(eng, ctrls, n_generate):
    """The same loop driven from Python through spec_draft / spec_verify / spec_accept / gammatune_update."""
    B = len(ctrls)
    gen = [0] * B
    steps, acc, drafted, gsum = 0, 0, 0, 0
    seq_steps = 0
    while min(gen) < n_generate:
        # a sequence that has its tokens rides along with gamma 1, uncounted, as in spec_generate
        gs = [c.gamma if gen[b] < n_generate else 1 for b, c in enumerate(ctrls)]
        eng.draft(gs[0] if B == 1 else np.array(gs, dtype=np.int32))
        eng.verify(max(gs))
        A, y, k = eng.accept()
        for b in range(B):
            if gen[b] >= n_generate:
                continue
            ctrls[b].update(int(A[b]), int(k[b]))
            gen[b] += int(A[b]) + 1
            acc += int(A[b])
            drafted += int(k[b])
            gsum += gs[b]
            seq_steps += 1
        steps += 1
    return dict(generated=sum(min(g, n_generate) for g in gen), spec_steps=steps, accepted=acc, drafted=drafted,
                gamma_sum=gsum, seq_steps=seq_steps)


def make_controller(pk, args, gamma_max):
    if args.controller == "fixed":
        return pk.FixedGamma(args.gamma0)
    return pk.GammaTune(eta=0.25, delta=1, gamma_min=1, gamma_max=gamma_max, gamma0=args.gamma0)


def cpu_model_name():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def esz_of(m):
    return {"bf16": 2, "q8": 1}.get(m.dtype, 4)


def proj_shapes(m):
    """(class id, name, output rows, K) of the weight-streaming launches of one layer and of the LM head; class ids
    are those of spec_profile_kernel."""
    qd, kvd = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    return [(1, "QKV", qd + 2 * kvd, m.d_model), (5, "Wo", m.d_model, qd), (3, "gate/up", 2 * m.d_ffn, m.d_model),
            (6, "down", m.d_model, m.d_ffn), (4, "LM head", m.vocab, m.d_model)]


def weight_bytes(m):
    per_layer = sum(n * k for cls, _, n, k in proj_shapes(m) if cls != 4)
    return (m.n_layers * per_layer + m.vocab * m.d_model) * esz_of(m)


def kv_bytes(m, context):
    """K and V of `context` positions over all layers (what one pass of one sequence attends to)."""
    return m.n_layers * 2 * m.n_kv_heads * m.head_dim * context * (4 if m.dtype == "fp32" else 2)


def kernel_table(eng, cfg, context, n_tokens, ctrls, decode):
    """Every kernel class of both models timed over one decode leg with direct launches: projections by the dispatch's
    own start / stop events, attention (+ merge) by events on the stream around its two launches.  Bytes are the
    algorithmic ones: the matrix once per launch; for attention the K and V of one layer at the leg's context."""
    eng.profile_kernel(0, 0)
    decode(eng, ctrls, n_tokens)
    rows = []
    for model, name, m in ((1, "target", cfg.target), (0, "draft", cfg.draft)):
        for cls, kname, n, k in proj_shapes(m):
            cnt, ms = eng.profile_read_class(model, cls)
            if cnt == 0:
                continue
            b = n * k * esz_of(m)
            us = 1e3 * ms / cnt
            rows.append({"model": name, "kernel": kname, "launches": cnt, "avg_us": us, "bytes": b,
                         "frac": b / (us * 1e-6) / 1e9 / HBM_PEAK_GBS})
        cnt, ms = eng.profile_read_class(model, 7)
        if cnt:
            b = kv_bytes(m, context) // m.n_layers
            us = 1e3 * ms / cnt
            rows.append({"model": name, "kernel": "attention + merge", "launches": cnt, "avg_us": us, "bytes": b,
                         "frac": b / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, "timing": "stream events around both launches"})
    eng.profile_read()
    eng.profile_kernel(0, -1)
    return rows


def verify_sweep(args, pk, torch, synth):
    """Verification passes alone (Experimental Details' largest Vicuna pair by shape unless --pair says otherwise):
    rows per sequence x cached positions x sequences, on a seeded synthetic cache; per cell the time of one pass
    (graph replay, host clock between two synchronisations over --sweep-reps passes) and its algorithmic bytes -
    every target weight once, the K / V the rows attend to, the logits written - against the HBM peak."""
    cfg = synth.pair(args.pair)
    m = cfg.target
    Wt, Wd = synth.make_pair_weights(synth.shrink(cfg, m.n_layers, 1), 0, device="cuda")
    torch.cuda.synchronize()
    rows_list = [int(x) for x in args.sweep_rows.split(",")]
    kv_list = [int(x) for x in args.sweep_kv.split(",")]
    b_list = [int(x) for x in args.sweep_batch.split(",")]
    gamma_max = max(max(rows_list) - 1, 1)
    cells = []
    for B in b_list:
        for kv in kv_list:
            eng = pk.SpecEngine(m, Wt, synth.shrink(cfg, m.n_layers, 1).draft, Wd, batch=B, max_seq=kv + 2 * gamma_max + 8,
                                gamma_max=gamma_max, temperature=1.0, seed=0, use_graphs=not args.no_graphs,
                                attn_chunk=args.attn_chunk)
            eng.fill_kv(kv)
            for rows in rows_list:
                for _ in range(3):
                    eng.verify_rows(rows)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(args.sweep_reps):
                    eng.verify_rows(rows)
                torch.cuda.synchronize()
                ms = 1e3 * (time.perf_counter() - t0) / args.sweep_reps
                nbytes = weight_bytes(m) + B * kv_bytes(m, kv + rows) + B * rows * m.vocab * 4
                gbs = nbytes / (ms * 1e-3) / 1e9
                # matrix-instruction work of the projections: 2 flop per weight and row, twice over (two bf16 terms of x)
                mfma_tflops = 2 * 2.0 * B * rows * (weight_bytes(m) / esz_of(m)) / (ms * 1e-3) / 1e12
                cells.append({"batch": B, "kv_len": kv, "rows_per_seq": rows, "rows": B * rows, "ms": ms, "bytes": nbytes,
                              "GB/s": gbs, "frac": gbs / HBM_PEAK_GBS, "mfma_tflops_issued": mfma_tflops,
                              "mfma_frac_of_peak": mfma_tflops / MFMA_BF16_PEAK_TFLOPS})
                print(f"# sweep batch {B} kv {kv} rows {rows}: {ms:.3f} ms {gbs:.0f} GB/s", file=sys.stderr, flush=True)
            eng.close()
    print(json.dumps({"verify_sweep": cells, "peak_GB/s": HBM_PEAK_GBS, "pair": args.pair,
                      "timing": "host clock around --sweep-reps spec_debug_verify_rows calls between two device synchronisations",
                      "config": {"workload": f"{args.pair} target {m.n_layers}L d{m.d_model} ffn{m.d_ffn} V{m.vocab}: verification "
                                             f"passes alone on a seeded synthetic KV cache"}}))


def cpu_baseline_full(cfg, Wt, Wd, gamma):
    """Two whole speculative steps of the fp64 oracle at full depth and width after a 32-token prompt."""
    import synth
    from oracle import gammatune as ogt
    from oracle import model as om
    from oracle import spec as ospec

    def oshape(ms):
        return om.Shape(ms.n_layers, ms.d_model, ms.n_q_heads, ms.n_kv_heads, ms.head_dim, ms.d_ffn, ms.vocab, ms.rope_theta,
                        ms.rms_eps, ms.dtype in ("bf16", "q8"))

    widen = lambda W: {k: ([om.as_f64(a) for a in v] if isinstance(v, list) else om.as_f64(v))
                       for k, v in synth.to_numpy_weights(W).items()}
    Wt_np, Wd_np = widen(Wt), widen(Wd)
    prompt = synth.make_prompts(1, 32, cfg.target.vocab, 11)[0].tolist()
    pair = ospec.TransformerPair(oshape(cfg.target), Wt_np, oshape(cfg.draft), Wd_np)
    scfg = ospec.StepConfig(temperature=0.7, seed=0, accept_mode=1, alpha=[0.6])
    toks = list(prompt)
    pair.target_rows(toks, 0)  # context, untimed
    pair.draft_next(toks)
    t0 = time.time()
    emitted = 0
    for s_ in range(2):
        r = ospec.speculative_step(pair.draft_next, pair.target_rows, toks, gamma, s_, 0, scfg, emitted)
        toks.extend(r.emitted)
        emitted += len(r.emitted)
    dt = time.time() - t0
    return {"value": emitted / dt, "unit": "tokens/s", "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)),
            "kind": "oracle", "cpu": cpu_model_name(),
            "sample": f"fp64 oracle, full depth and width: two whole speculative steps (gamma {gamma}, forced alpha 0.6) after a "
                      f"32-token context, {emitted} tokens in {dt:.1f} s"}


def cpu_baseline(cfg, Wt, Wd, tokens_per_step, mean_gamma):
    """Time the fp64 oracle at full width on a bounded sample and extrapolate over the layers."""
    import synth
    from oracle import model as om

    def oshape(ms, L):
        return om.Shape(L, ms.d_model, ms.n_q_heads, ms.n_kv_heads, ms.head_dim, ms.d_ffn, ms.vocab, ms.rope_theta,
                        ms.rms_eps, ms.dtype in ("bf16", "q8"))

    def host(W, L):
        # widened to fp64 once, outside the timed region, as the full-width parity tests hand them to the oracle (the
        # oracle also takes bf16 bit patterns and widens them per use: 20 x slower, and not what is timed here)
        Wn = synth.to_numpy_weights({k: (v[:L] if isinstance(v, list) else v) for k, v in W.items()})
        return {k: ([om.as_f64(a) for a in v] if isinstance(v, list) else om.as_f64(v)) for k, v in Wn.items()}

    prompt = synth.make_prompts(1, 32, cfg.target.vocab, 11)[0]
    gamma = max(1, int(round(mean_gamma)))
    out = {}
    t_all0 = time.time()
    for name, ms, W, Ls, rows in (("target", cfg.target, Wt, (0, 1), gamma + 1), ("draft", cfg.draft, Wd, (0, 1), 1)):
        t = {}
        for L in Ls:
            Wn = host(W, L)
            cache = om.KVCache(oshape(ms, L))
            om.forward(oshape(ms, L), Wn, prompt, cache)         # context, untimed
            t0 = time.time()
            om.forward(oshape(ms, L), Wn, prompt[:rows], cache)  # the timed rows
            t[L] = time.time() - t0
        per_layer = max(t[1] - t[0], 0.0)
        out[name] = t[0] + per_layer * ms.n_layers
    step_s = gamma * out["draft"] + out["target"]
    return {
        "value": tokens_per_step / step_s,
        "unit": "tokens/s",
        "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)),
        "kind": "oracle",
        "cpu": cpu_model_name(),
        "sample": (f"fp64 oracle on weights widened to fp64 beforehand, full width: one {gamma + 1}-row target pass and one 1-row draft pass after a 32-token "
                   f"context, timed with 0 and 1 layers (+ embedding, final norm, LM head) and extrapolated linearly to "
                   f"{cfg.target.n_layers}/{cfg.draft.n_layers} layers; step = {gamma} draft passes + 1 target pass, "
                   f"{tokens_per_step:.2f} tokens per step as measured on the GPU run; sample took {time.time() - t_all0:.1f} s"),
    }


TRAFFIC_FILE = os.path.join(ROOT, "profiles", "gemv_gate_up_8b_pmc.json")
KERNEL_SOURCES = ["gemv_mfma.hip", "epilogue.hpp", "common.hpp", "kv.hpp", "q8.hpp"]  # the files that hold the kernel's code
COPY_BYTES = 1 << 30


def kernel_source_digest():
    """Digest of the roofline kernel's code: its source files with comments and white space removed."""
    import hashlib
    import re
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2504_00030_amd", "csrc", "kernels", name), "r") as f:
            text = f.read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        text = re.sub(r"//[^\n]*", "", text)
        h.update("".join(text.split()).encode())
    return h.hexdigest()


def measured_traffic(pair):
    """HBM bytes per launch of the roofline kernel from stored profiler counters (FETCH_SIZE and WRITE_SIZE, KiB per
    dispatch), each scaled by what the same counter read for the plain copy of COPY_BYTES in the same run.  None when
    no counters are stored, or when the kernel's sources changed after they were taken."""
    if pair != "8b" or not os.path.exists(TRAFFIC_FILE):
        return None
    with open(TRAFFIC_FILE) as f:
        t = json.load(f)
    if t.get("source_sha256") != kernel_source_digest():
        return None
    fetch = t["kernel_fetch_kib"] * 1024.0 * (t["copy_bytes"] / (t["copy_fetch_kib"] * 1024.0))
    write = t["kernel_write_kib"] * 1024.0 * (t["copy_bytes"] / (t["copy_write_kib"] * 1024.0))
    return fetch + write


def main():
    args = parse()
    if args.host_loop:
        globals()["decode_loop"] = decode_loop_host
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import synth
    import paper_2504_00030_amd as pk

    pk.load()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.verify_sweep:
        verify_sweep(args, pk, torch, synth)
        return
    cfg = synth.pair(args.pair)
    n_gen = args.n_generate or cfg.n_generate
    n_prompt = args.prompt_len or cfg.prompt_len
    t0 = time.time()
    Wt, Wd = synth.make_pair_weights(cfg, 0, device="cuda")
    torch.cuda.synchronize()
    t_weights = time.time() - t0

    if args.alpha == "piecewise":
        alpha = synth.alpha_piecewise(n_gen + 64, 32, 0.9, 0.3)
    else:
        alpha = synth.alpha_constant(float(args.alpha), 4)
    tau = float(np.float32(0.4)) if args.controller == "gammatune+" else 0.0
    # with several sequences the fast ones ride along (gamma 1: at most two tokens per step) until the slowest has
    # n_gen tokens, which takes at most n_gen steps: 3 n_gen tokens of room is the worst case
    max_seq = n_prompt + n_gen * (1 if args.batch == 1 else 3) + 2 * cfg.gamma_max + 8
    B = args.batch
    prompts = synth.make_prompts(B, n_prompt, cfg.target.vocab, 7)

    forced = args.accept == "forced"

    def engine(use_graphs, early_stop=True):
        e = pk.SpecEngine(cfg.target, Wt, cfg.draft, Wd, batch=B, max_seq=max_seq, gamma_max=cfg.gamma_max,
                          temperature=args.temperature, seed=0, accept_mode=pk.ACCEPT_FORCED if forced else pk.ACCEPT_NATURAL,
                          use_graphs=use_graphs, gemv_path=args.gemv_path, attn_chunk=args.attn_chunk)
        if forced:
            e.set_forced_alpha(alpha)
        if tau > 0 and early_stop:
            e.set_early_stop(tau)
        return e

    def prefill_report(seconds):
        """Prompt ingestion: every sequence's first n_prompt - 1 tokens through both models (the last prompt token
        enters with the first speculative step).  `achieved` counts the projections' useful flops, 2 x rows x
        weights; the kernel multiplies each weight by both bf16 terms of the activation, twice that many
        matrix-instruction flops.  Attention, embedding and the epilogues are inside the time, not the flops."""
        rows = B * (n_prompt - 1)
        def proj_weights(m):
            qd, kvd = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
            return m.n_layers * (m.d_model * (qd + 2 * kvd) + qd * m.d_model + 3 * m.d_model * m.d_ffn)
        flops = 2.0 * rows * (proj_weights(cfg.target) + proj_weights(cfg.draft))
        tf = flops / seconds / 1e12 if seconds > 0 else 0.0
        return {"ms": 1e3 * seconds, "rows": rows, "tokens_per_s": rows / seconds if seconds > 0 else 0.0,
                "bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": tf / MFMA_BF16_PEAK_TFLOPS, "matrix_instruction_flops_per_useful_flop": 2}

    if args.prefill_only:
        eng = engine(not args.no_graphs)
        for _ in range(args.warmup):
            eng.prefill(prompts)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            eng.prefill(prompts)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / max(args.steps, 1)
        eng.close()
        print(json.dumps({"prefill": prefill_report(dt), "steps": args.steps, "warmup": args.warmup,
                          "config": {"workload": f"{args.pair}: batch {B}, prompt {n_prompt}"}}))
        return
    if args.roofline_only:
        args.warmup = args.steps = 0
    eng = engine(not args.no_graphs)
    stats = dict(generated=0, spec_steps=0, accepted=0, drafted=0, gamma_sum=0)
    t_prefill = 0.0
    for _ in range(args.warmup):
        eng.prefill(prompts)
        decode_loop(eng, [make_controller(pk, args, cfg.gamma_max) for _ in range(B)], n_gen)
    total = 0.0
    for _ in range(args.steps):
        torch.cuda.synchronize()
        tp = time.perf_counter()
        eng.prefill(prompts)
        torch.cuda.synchronize()
        t_prefill += time.perf_counter() - tp
        ctrl = [make_controller(pk, args, cfg.gamma_max) for _ in range(B)]
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        stats = decode_loop(eng, ctrl, n_gen)
        torch.cuda.synchronize()
        total += time.perf_counter() - t1
    steps = max(args.steps, 1)
    tok_s = steps * B * n_gen / total if total > 0 else 0.0
    eng.close()

    roofline = None
    if not args.skip_roofline:
        e2 = engine(False)
        e2.prefill(prompts)
        e2.profile_kernel(1, 3)  # target model, gate/up projection + SwiGLU
        c2 = [make_controller(pk, args, cfg.gamma_max) for _ in range(B)]
        decode_loop(e2, c2, min(n_gen, 32 if args.roofline_only else 128))
        n_launch, ms = e2.profile_read()
        e2.close()
        # reference traffic for profiler byte counters: one plain copy of known size
        src = torch.empty(COPY_BYTES, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        pk.k_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst
        bytes_per_launch = 2 * cfg.target.d_ffn * cfg.target.d_model * {"bf16": 2, "q8": 1}.get(cfg.target.dtype, 4)
        avg_ms = ms / max(n_launch, 1)
        achieved = bytes_per_launch / (avg_ms * 1e-3) / 1e9 if avg_ms > 0 else 0.0
        traffic = measured_traffic(args.pair)
        roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "kernel": "target gate/up projection + SwiGLU",
                    "launches": n_launch, "avg_us": avg_ms * 1e3, "bytes_per_launch": bytes_per_launch,
                    "timing": "hip events of the dispatch (kernel start to kernel end), averaged over every launch of the "
                              "kernel in a decode leg of this run with direct launches",
                    "traffic_source": (None if traffic is None else
                                       "stored rocprofv3 FETCH_SIZE / WRITE_SIZE passes (profiles/gemv_gate_up_8b_pmc.json), "
                                       "not measured in this run; nulled when the kernel's sources change")}

    verify_pass = None
    if not args.skip_roofline and B == 1:
        # the whole verification pass against the HBM roofline: gamma = 2 (the run's mean), graphs, one
        # synchronisation on either side of spec_verify; bytes = every target weight once + the visible KV cache
        e3 = engine(not args.no_graphs)
        e3.prefill(prompts)
        g, n_pass, t_ver = 2, 48, 0.0
        for i in range(n_pass + 4):
            e3.draft(g)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            e3.verify(g)
            torch.cuda.synchronize()
            if i >= 4:
                t_ver += time.perf_counter() - t0
            e3.accept()
        e3.close()
        m = cfg.target
        qd, kvd = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
        esz = {"bf16": 2, "q8": 1}.get(m.dtype, 4)
        w_bytes = weight_bytes(m)
        kv_b = kv_bytes(m, n_prompt + n_pass)  # context at the middle of the leg, roughly
        ms = 1e3 * t_ver / n_pass
        gbs = (w_bytes + kv_b) / (ms * 1e-3) / 1e9
        verify_pass = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                       "ms": ms, "bytes": w_bytes + kv_b, "gamma": g, "passes": n_pass,
                       "timing": "host clock around spec_verify between two device synchronisations"}

    draft_pass = None
    kernels = None
    if not args.skip_roofline and B == 1:
        # one draft-model decode pass against the HBM roofline: a fixed gamma = 3 without early stopping is one graph
        # of three passes (the first ingests the one or two pending rows); bytes = every draft weight once + its KV
        e4 = engine(not args.no_graphs, early_stop=False)
        e4.prefill(prompts)
        g, n_rep, t_dr = 3, 48, 0.0
        for i in range(n_rep + 4):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            e4.draft(g)
            torch.cuda.synchronize()
            if i >= 4:
                t_dr += time.perf_counter() - t0
            e4.verify(g)
            e4.accept()
        e4.close()
        md = cfg.draft
        d_bytes = weight_bytes(md) + kv_bytes(md, n_prompt + n_rep)
        ms = 1e3 * t_dr / (n_rep * g)
        gbs = d_bytes / (ms * 1e-3) / 1e9
        draft_pass = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                      "ms": ms, "bytes": d_bytes, "gamma": g, "passes": n_rep * g,
                      "timing": "host clock around spec_draft (one graph of gamma passes with their samplers) between two "
                                "device synchronisations, divided by gamma"}
        # every kernel class of both models over one decode leg (direct launches)
        e5 = engine(False)
        e5.prefill(prompts)
        kernels = kernel_table(e5, cfg, n_prompt + 32, 64, [make_controller(pk, args, cfg.gamma_max) for _ in range(B)],
                               decode_loop)
        e5.close()

    seq_steps = max(stats.get("seq_steps", stats["spec_steps"]), 1)  # (sequence, speculative step) pairs
    tokens_per_step = stats["generated"] / seq_steps
    mean_gamma = stats["gamma_sum"] / seq_steps
    cpu = None
    if not args.skip_cpu:
        cpu = (cpu_baseline_full(cfg, Wt, Wd, max(1, int(round(mean_gamma)))) if args.cpu_full
               else cpu_baseline(cfg, Wt, Wd, tokens_per_step, mean_gamma))

    line = {
        "metric": ("generated tokens/s (8B-shaped pair, bs1); verify-pass HBM GB/s % of peak" if (args.pair == "8b" and B == 1)
                   else f"generated tokens/s ({args.pair} pair, bs{B})"),
        "value": tok_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * total / steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.target.dtype == "q8" else cfg.target.dtype, "data": "synthetic",
        "config": {
            "workload": (f"{args.pair}: target {cfg.target.n_layers}L d{cfg.target.d_model} ffn{cfg.target.d_ffn} "
                         f"V{cfg.target.vocab}, draft {cfg.draft.n_layers}L d{cfg.draft.d_model}; batch {B}, prompt {n_prompt}, "
                         f"generate {n_gen}; {args.controller} gamma in [1,{cfg.gamma_max}] gamma0 {args.gamma0}, "
                         f"T={args.temperature}, " + (f"forced alpha {args.alpha}" if forced else "natural acceptance")
                         + f", tau {tau}; seeded random-init weights"
                         + ("; projection matrices and LM head int8 with per-row scales, turned into bf16 in registers"
                            if cfg.target.dtype == "q8" else "")),
            "step": f"one generation of {n_gen} tokens (prefill excluded)",
            "graphs": not args.no_graphs, "spec_steps": stats["spec_steps"], "tokens_per_spec_step": tokens_per_step,
            "mean_gamma": mean_gamma, "mean_accepted": stats["accepted"] / seq_steps,
            "mean_drafted": stats["drafted"] / seq_steps,
            "prefill_ms": 1e3 * t_prefill / steps, "weights_s": t_weights,
        },
        "roofline": roofline, "cpu_baseline": cpu,
        "prefill": prefill_report(t_prefill / steps) if args.steps > 0 else None,
        "verify_pass": verify_pass, "draft_pass": draft_pass, "kernels": kernels,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
