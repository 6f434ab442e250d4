"""Llama-style decoder forward in fp64: the draft and target models of the
speculative step (Background section: a small draft model proposes tokens
autoregressively, the large target model scores them in one parallel pass).

Test infrastructure only (see oracle/__init__.py).

The paper names checkpoints only; the architecture conventions below are the
ones both sides implement independently:
  * RMSNorm: y = x * rsqrt(mean(x^2) + eps) * g
  * RoPE, rotate-half pairing: element j pairs with j + hd/2, angle
    pos * theta**(-2j/hd); no frequency rescaling
  * attention: softmax(q k^T / sqrt(hd)) v with a causal mask on absolute
    positions; query head h reads kv head h // (n_q / n_kv)
  * MLP: W_down( silu(W_gate m) * (W_up m) ), no biases
  * with kv_bf16 the rotated K and V are rounded to bfloat16 (nearest even)
    when they are written to the cache, because the 16-bit cache is a data
    format, like the 16-bit weights (Experimental Details: weights and KV
    cache are kept in 16-bit floating point)

Weights may be float32 / float64 arrays or uint16 arrays holding bfloat16
bit patterns; all arithmetic is float64.  Results are defined by the full
prefix; the cache is only a way of not recomputing rows and `forward` with a
cache must equal one call over the whole sequence.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional

import numpy as np


@dataclass
class Shape:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_theta: float = 10000.0
    rms_eps: float = 1e-5
    kv_bf16: bool = False


def as_f64(a: np.ndarray) -> np.ndarray:
    """float view of a weight array; uint16 is read as bfloat16 bit patterns."""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return np.asarray(a, dtype=np.float64)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bfloat16 (ties to even), return as float64."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    bits = (bits + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    return bits.astype(np.uint32).view(np.float32).astype(np.float64)


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def rope(v: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """v: [n, heads, hd]; pos: [n] absolute positions."""
    hd = v.shape[-1]
    half = hd // 2
    j = np.arange(half, dtype=np.float64)
    inv_freq = theta ** (-2.0 * j / hd)
    ang = pos.astype(np.float64)[:, None] * inv_freq[None, :]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    a, b = v[..., :half], v[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


class KVCache:
    """Per-layer lists of rotated keys and values, [len, n_kv, hd] each."""

    def __init__(self, shape: Shape):
        self.k: List[np.ndarray] = [np.zeros((0, shape.n_kv_heads, shape.head_dim)) for _ in range(shape.n_layers)]
        self.v: List[np.ndarray] = [np.zeros((0, shape.n_kv_heads, shape.head_dim)) for _ in range(shape.n_layers)]
        self.length = 0

    def truncate(self, n: int) -> None:
        self.k = [a[:n] for a in self.k]
        self.v = [a[:n] for a in self.v]
        self.length = min(self.length, n)


def forward(shape: Shape, W: Dict, tokens, cache: Optional[KVCache] = None) -> np.ndarray:
    """Logits [n, vocab] (float64) for `tokens` appended after the cached prefix.

    W keys: tok_embed [V,d], lm_head [V,d], final_norm [d], and per-layer lists
    wq [nq*hd,d], wk, wv [nkv*hd,d], wo [d,nq*hd], w_gate, w_up [ffn,d],
    w_down [d,ffn], attn_norm [d], ffn_norm [d].
    """
    tokens = np.asarray(tokens, dtype=np.int64).reshape(-1)
    n = tokens.shape[0]
    if cache is None:
        cache = KVCache(shape)
    pos0 = cache.length
    pos = pos0 + np.arange(n)
    nq, nkv, hd = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    group = nq // nkv

    h = as_f64(W["tok_embed"][tokens])
    for l in range(shape.n_layers):
        a = rmsnorm(h, as_f64(W["attn_norm"][l]), shape.rms_eps)
        q = (a @ as_f64(W["wq"][l]).T).reshape(n, nq, hd)
        k = (a @ as_f64(W["wk"][l]).T).reshape(n, nkv, hd)
        v = (a @ as_f64(W["wv"][l]).T).reshape(n, nkv, hd)
        q = rope(q, pos, shape.rope_theta)
        k = rope(k, pos, shape.rope_theta)
        if shape.kv_bf16:
            k = round_bf16(k)
            v = round_bf16(v)
        cache.k[l] = np.concatenate([cache.k[l][:pos0], k], axis=0)
        cache.v[l] = np.concatenate([cache.v[l][:pos0], v], axis=0)
        K, V = cache.k[l], cache.v[l]
        total = pos0 + n
        allowed = np.arange(total)[None, :] <= pos[:, None]
        o = np.empty((n, nq, hd))
        for hq in range(nq):
            kvh = hq // group
            sc = (q[:, hq, :] @ K[:, kvh, :].T) / np.sqrt(float(hd))
            sc = np.where(allowed, sc, -np.inf)
            sc = sc - sc.max(axis=-1, keepdims=True)
            p = np.exp(sc)
            p = p / p.sum(axis=-1, keepdims=True)
            o[:, hq, :] = p @ V[:, kvh, :]
        h = h + o.reshape(n, nq * hd) @ as_f64(W["wo"][l]).T
        m = rmsnorm(h, as_f64(W["ffn_norm"][l]), shape.rms_eps)
        act = silu(m @ as_f64(W["w_gate"][l]).T) * (m @ as_f64(W["w_up"][l]).T)
        h = h + act @ as_f64(W["w_down"][l]).T
    cache.length = pos0 + n
    hf = rmsnorm(h, as_f64(W["final_norm"]), shape.rms_eps)
    return hf @ as_f64(W["lm_head"]).T
