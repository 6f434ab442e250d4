"""Seeded random-init weights, N(0, 0.02^2), as torch tensors on any device.

The same tensors feed both sides: the GPU library gets their device pointers,
the CPU oracle gets numpy copies (`to_numpy_weights`; bf16 travels as its
uint16 bit pattern).  Values depend on (seed, device type): generate once and
copy, never generate separately per side.
"""
from __future__ import annotations

from typing import Dict

import numpy as np
import torch

from .configs import ModelShape, PairConfig

STD = 0.02


def _dtype(shape: ModelShape):
    # "q8" models keep embedding, norms and KV cache in bf16; their matrices are quantised by quantize_weights
    return torch.float32 if shape.dtype == "fp32" else torch.bfloat16


MATRICES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


def quantize_rows(w: torch.Tensor):
    """Symmetric 8-bit weights with one fp32 scale per output row: w ~ scale[n] * q[n][k], q in [-127, 127].
    The quantised model is DEFINED by (q, scale); how they were obtained from a random matrix is immaterial."""
    q = torch.empty(w.shape, dtype=torch.int8, device=w.device)
    scale = torch.empty(w.shape[0], dtype=torch.float32, device=w.device)
    step = max(1, (1 << 26) // max(w.shape[1], 1))
    for r0 in range(0, w.shape[0], step):
        blk = w[r0:r0 + step].float()
        sc = blk.abs().amax(dim=1).clamp_min(1e-12) / 127.0
        scale[r0:r0 + step] = sc
        q[r0:r0 + step] = torch.round(blk / sc[:, None]).clamp_(-127, 127).to(torch.int8)
    return q, scale


def quantize_weights(W: Dict) -> Dict:
    """The projection matrices and the LM head of W as (int8, per-row fp32 scale) pairs: key k holds q, key
    k + "_scale" the scales.  Embedding and norm weights stay as they are."""
    out = dict(W)
    for k in MATRICES:
        qs = [quantize_rows(w) for w in W[k]]
        out[k] = [q for q, _ in qs]
        out[k + "_scale"] = [s for _, s in qs]
    out["lm_head"], out["lm_head_scale"] = quantize_rows(W["lm_head"])
    return out


def _normal(gen, rows, cols, dtype, device, std=STD):
    # generated in fp32 in row blocks so that a large matrix never needs a second full-size temporary
    out = torch.empty((rows, cols), dtype=dtype, device=device)
    step = max(1, (1 << 26) // max(cols, 1))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        blk = torch.randn((r1 - r0, cols), generator=gen, device=device, dtype=torch.float32) * std
        out[r0:r1] = blk.to(dtype)
    return out


def make_weights(shape: ModelShape, seed: int, device="cpu", norm_jitter: float = 0.0, tied_head: bool = False) -> Dict:
    """Dict with tok_embed, lm_head, final_norm and per-layer lists wq, wk, wv, wo,
    w_gate, w_up, w_down, attn_norm, ffn_norm.  Norm weights are 1 (+ jitter*N(0,1) for tests)."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(int(seed))
    dt = _dtype(shape)
    d, hd = shape.d_model, shape.head_dim
    nq, nkv, ffn, V = shape.n_q_heads, shape.n_kv_heads, shape.d_ffn, shape.vocab

    def norm_w():
        w = torch.ones(d, dtype=torch.float32, device=dev)
        if norm_jitter:
            w = w + norm_jitter * torch.randn(d, generator=gen, device=dev, dtype=torch.float32)
        return w.to(dt)

    W: Dict = {k: [] for k in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "attn_norm", "ffn_norm")}
    W["tok_embed"] = _normal(gen, V, d, dt, dev)
    for _ in range(shape.n_layers):
        W["wq"].append(_normal(gen, nq * hd, d, dt, dev))
        W["wk"].append(_normal(gen, nkv * hd, d, dt, dev))
        W["wv"].append(_normal(gen, nkv * hd, d, dt, dev))
        W["wo"].append(_normal(gen, d, nq * hd, dt, dev))
        W["w_gate"].append(_normal(gen, ffn, d, dt, dev))
        W["w_up"].append(_normal(gen, ffn, d, dt, dev))
        W["w_down"].append(_normal(gen, d, ffn, dt, dev))
        W["attn_norm"].append(norm_w())
        W["ffn_norm"].append(norm_w())
    W["final_norm"] = norm_w()
    W["lm_head"] = W["tok_embed"] if tied_head else _normal(gen, V, d, dt, dev)
    return W


def make_pair_weights(cfg: PairConfig, seed: int, device="cpu", norm_jitter: float = 0.0):
    """(target weights, draft weights) for a pair; see PairConfig.draft_kind."""
    if cfg.draft_kind == "prefix":
        Wt = make_weights(cfg.target, seed, device, norm_jitter, tied_head=True)
        n = cfg.draft.n_layers
        Wd = {k: (v[:n] if isinstance(v, list) else v) for k, v in Wt.items()}
        return Wt, Wd
    Wt = make_weights(cfg.target, seed, device, norm_jitter)
    Wd = make_weights(cfg.draft, seed + 1, device, norm_jitter)
    if cfg.draft_kind == "projected_head":
        # draft head = target head times a random [d_draft, d_target] projection, entries N(0, 1/d_target)
        dev = torch.device(device)
        gen = torch.Generator(device=dev)
        gen.manual_seed(int(seed) + 2)
        dt_, dd_ = cfg.target.d_model, cfg.draft.d_model
        P = torch.randn((dd_, dt_), generator=gen, device=dev, dtype=torch.float32) * (dt_ ** -0.5)
        head = torch.empty((cfg.draft.vocab, dd_), dtype=Wd["lm_head"].dtype, device=dev)
        step = 16384
        for r0 in range(0, cfg.draft.vocab, step):
            head[r0:r0 + step] = (Wt["lm_head"][r0:r0 + step].float() @ P.t()).to(head.dtype)
        Wd["lm_head"] = head
    if cfg.target.dtype == "q8":
        Wt = quantize_weights(Wt)
    if cfg.draft.dtype == "q8":
        Wd = quantize_weights(Wd)
    return Wt, Wd


def _np(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def to_numpy_weights(W: Dict) -> Dict:
    """Host numpy copy for the oracle (bf16 -> uint16 bit patterns).  Quantised matrices (int8 with a "_scale"
    partner) come out as the fp64 matrices they stand for, scale[n] * q[n][k], and the scale keys are dropped."""
    out = {}
    for k, v in W.items():
        if k.endswith("_scale"):
            continue
        sc = W.get(k + "_scale")
        if sc is None:
            out[k] = [_np(t) for t in v] if isinstance(v, list) else _np(v)
        elif isinstance(v, list):
            out[k] = [_np(s).astype(np.float64)[:, None] * _np(q).astype(np.float64) for q, s in zip(v, sc)]
        else:
            out[k] = _np(sc).astype(np.float64)[:, None] * _np(v).astype(np.float64)
    return out
