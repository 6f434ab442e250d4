"""Pins for oracle.model and the generate loop: a second forward assembled from torch CPU ops,
structural invariants, and greedy speculative == greedy target-only (Background section)."""
import math
from dataclasses import replace

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth
from oracle import gammatune as gt
from oracle import model as om
from oracle import spec


def oshape(ms: synth.ModelShape) -> om.Shape:
    return om.Shape(ms.n_layers, ms.d_model, ms.n_q_heads, ms.n_kv_heads, ms.head_dim, ms.d_ffn, ms.vocab,
                    ms.rope_theta, ms.rms_eps, ms.dtype == "bf16")


def torch_forward(ms: synth.ModelShape, W, tokens, round_kv=False):
    """Independent formulation: F.linear / F.scaled_dot_product_attention, RoPE as complex rotation."""
    f64 = lambda t: t.to(torch.float64)
    n = len(tokens)
    nq, nkv, hd = ms.n_q_heads, ms.n_kv_heads, ms.head_dim
    h = f64(W["tok_embed"])[torch.as_tensor(tokens, dtype=torch.long)]
    pos = torch.arange(n, dtype=torch.float64)
    inv = 1.0 / (ms.rope_theta ** (torch.arange(0, hd, 2, dtype=torch.float64) / hd))
    rot = torch.polar(torch.ones(n, hd // 2, dtype=torch.float64), pos[:, None] * inv[None, :])  # e^{i*angle}

    def rms(x, g):
        return x * torch.rsqrt(x.pow(2).mean(-1, keepdim=True) + ms.rms_eps) * f64(g)

    def rope(x):  # x [n, H, hd], pairs (j, j+hd/2)
        z = torch.complex(x[..., : hd // 2], x[..., hd // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    def bf(x):
        return x.to(torch.float32).to(torch.bfloat16).to(torch.float64) if round_kv else x

    for l in range(ms.n_layers):
        a = rms(h, W["attn_norm"][l])
        q = rope(F.linear(a, f64(W["wq"][l])).view(n, nq, hd))
        k = bf(rope(F.linear(a, f64(W["wk"][l])).view(n, nkv, hd)))
        v = bf(F.linear(a, f64(W["wv"][l])).view(n, nkv, hd))
        k = k.repeat_interleave(nq // nkv, dim=1)
        v = v.repeat_interleave(nq // nkv, dim=1)
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None], v.transpose(0, 1)[None],
                                           is_causal=True)[0].transpose(0, 1).reshape(n, nq * hd)
        h = h + F.linear(o, f64(W["wo"][l]))
        m = rms(h, W["ffn_norm"][l])
        h = h + F.linear(F.silu(F.linear(m, f64(W["w_gate"][l]))) * F.linear(m, f64(W["w_up"][l])), f64(W["w_down"][l]))
    return F.linear(rms(h, W["final_norm"]), f64(W["lm_head"])).numpy()


SMALL_GQA = synth.ModelShape(3, 96, 6, 2, 16, 200, 97, 500000.0, 1e-5, "fp32")
SMALL_BF16 = synth.ModelShape(2, 64, 4, 2, 16, 96, 61, 10000.0, 1e-5, "bf16")


@pytest.mark.parametrize("ms", [synth.pair("tiny").target, SMALL_GQA], ids=["tiny", "gqa"])
def test_forward_matches_torch_composition(ms):
    W = synth.make_weights(ms, 5, norm_jitter=0.1)
    Wn = synth.to_numpy_weights(W)
    toks = synth.make_prompts(1, 24, ms.vocab, 2)[0]
    got = om.forward(oshape(ms), Wn, toks)
    want = torch_forward(ms, W, toks)
    assert got.shape == (24, ms.vocab)
    assert np.max(np.abs(got - want)) < 1e-10 * max(1.0, np.abs(want).max())


def test_forward_bf16_weights_and_kv_rounding():
    ms = SMALL_BF16
    W = synth.make_weights(ms, 6, norm_jitter=0.1)
    Wn = synth.to_numpy_weights(W)
    assert Wn["wq"][0].dtype == np.uint16
    toks = synth.make_prompts(1, 12, ms.vocab, 3)[0]
    got = om.forward(oshape(ms), Wn, toks)
    want = torch_forward(ms, W, toks, round_kv=True)
    # both round K and V to bf16; a value within an fp64 ulp of a rounding boundary may flip, hence 1e-3 not 1e-10
    assert np.max(np.abs(got - want)) < 1e-3 * np.abs(want).max()
    # rounding matters: without it the result differs visibly
    plain = torch_forward(ms, W, toks, round_kv=False)
    assert np.max(np.abs(plain - want)) > 1e-6 * np.abs(want).max()


def test_round_bf16_matches_torch():
    x = np.random.default_rng(0).standard_normal(4096) * np.logspace(-8, 8, 4096)
    got = om.round_bf16(x)
    want = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(got, want)
    bits = np.array([0x3F80, 0x4000, 0xBF80, 0x0000], dtype=np.uint16)
    assert np.array_equal(om.as_f64(bits), [1.0, 2.0, -1.0, 0.0])


def test_cached_equals_one_shot():
    ms = SMALL_GQA
    Wn = synth.to_numpy_weights(synth.make_weights(ms, 7, norm_jitter=0.1))
    sh = oshape(ms)
    toks = synth.make_prompts(1, 20, ms.vocab, 4)[0]
    full = om.forward(sh, Wn, toks)
    cache = om.KVCache(sh)
    parts = [om.forward(sh, Wn, toks[:7], cache), om.forward(sh, Wn, toks[7:8], cache), om.forward(sh, Wn, toks[8:], cache)]
    assert np.max(np.abs(np.concatenate(parts) - full)) < 1e-11
    # truncating and re-feeding rewrites the same rows
    cache.truncate(10)
    again = om.forward(sh, Wn, toks[10:], cache)
    assert np.max(np.abs(again - full[10:])) < 1e-11


def test_rope_depends_on_relative_position_only():
    rng = np.random.default_rng(1)
    q = rng.standard_normal((5, 2, 16))
    k = rng.standard_normal((5, 2, 16))
    pos = np.arange(5)
    s0 = np.einsum("ihd,jhd->hij", om.rope(q, pos, 10000.0), om.rope(k, pos, 10000.0))
    s1 = np.einsum("ihd,jhd->hij", om.rope(q, pos + 37, 10000.0), om.rope(k, pos + 37, 10000.0))
    assert np.max(np.abs(s0 - s1)) < 1e-10
    # position 0 is the identity; norms are preserved
    assert np.allclose(om.rope(q, np.zeros(5, dtype=int), 10000.0), q)
    assert np.allclose(np.linalg.norm(om.rope(q, pos, 10000.0), axis=-1), np.linalg.norm(q, axis=-1))
    # pairing is (j, j + hd/2): rotating e_0 moves weight to element hd/2, angle = pos for j = 0
    e0 = np.zeros((1, 1, 16)); e0[0, 0, 0] = 1.0
    r = om.rope(e0, np.array([1]), 10000.0)[0, 0]
    assert r[0] == pytest.approx(math.cos(1.0)) and r[8] == pytest.approx(math.sin(1.0))
    assert np.count_nonzero(np.abs(r) > 1e-15) == 2


def test_rmsnorm_scale_invariance_and_silu():
    x = np.random.default_rng(2).standard_normal((3, 64))
    g = np.ones(64)
    assert np.allclose(om.rmsnorm(7.0 * x, g, 0.0), om.rmsnorm(x, g, 0.0))
    assert np.allclose((om.rmsnorm(x, g, 0.0) ** 2).mean(-1), 1.0)
    assert om.silu(np.array([0.0]))[0] == 0.0
    assert om.silu(np.array([1.0]))[0] == pytest.approx(1.0 / (1.0 + math.exp(-1.0)))


def test_gqa_with_replicated_kv_heads_equals_mha():
    ms = SMALL_GQA
    W = synth.to_numpy_weights(synth.make_weights(ms, 8))
    toks = synth.make_prompts(1, 10, ms.vocab, 5)[0]
    got = om.forward(oshape(ms), W, toks)
    rep = ms.n_q_heads // ms.n_kv_heads
    hd = ms.head_dim
    W2 = dict(W)
    W2["wk"] = [np.repeat(w.reshape(ms.n_kv_heads, hd, -1), rep, axis=0).reshape(ms.n_q_heads * hd, -1) for w in W["wk"]]
    W2["wv"] = [np.repeat(w.reshape(ms.n_kv_heads, hd, -1), rep, axis=0).reshape(ms.n_q_heads * hd, -1) for w in W["wv"]]
    mha = replace(oshape(ms), n_kv_heads=ms.n_q_heads)
    assert np.max(np.abs(om.forward(mha, W2, toks) - got)) < 1e-11


def test_prefix_draft_is_truncated_target():
    cfg = synth.pair("tiny")
    Wt, Wd = synth.make_pair_weights(cfg, 0)
    assert len(Wd["wq"]) == 2 and Wd["lm_head"] is Wt["tok_embed"]
    Wtn, Wdn = synth.to_numpy_weights(Wt), synth.to_numpy_weights(Wd)
    toks = synth.make_prompts(1, 9, cfg.target.vocab, 1)[0]
    d = om.forward(oshape(cfg.draft), Wdn, toks)
    Wcut = {k: (v[:2] if isinstance(v, list) else v) for k, v in Wtn.items()}
    assert np.array_equal(d, om.forward(oshape(replace(cfg.target, n_layers=2)), Wcut, toks))
    assert not np.allclose(d, om.forward(oshape(cfg.target), Wtn, toks))


@pytest.mark.parametrize("ctrl", ["fixed1", "fixed4", "gammatune"])
def test_greedy_speculative_equals_greedy_target_only(ctrl):
    cfg = synth.pair("tiny")
    Wt, Wd = synth.make_pair_weights(cfg, 0)
    Wtn, Wdn = synth.to_numpy_weights(Wt), synth.to_numpy_weights(Wd)
    prompt = synth.make_prompts(1, 12, cfg.target.vocab, 7)[0].tolist()
    pairm = spec.TransformerPair(oshape(cfg.target), Wtn, oshape(cfg.draft), Wdn)
    c = {"fixed1": gt.FixedGamma(1), "fixed4": gt.FixedGamma(4),
         "gammatune": gt.Controller(gt.Params(gamma_max=8), 4)}[ctrl]
    scfg = spec.StepConfig(temperature=0.0)
    res = spec.generate(pairm.draft_next, pairm.target_rows, prompt, 24, c, scfg)
    ref_pair = spec.TransformerPair(oshape(cfg.target), Wtn, oshape(cfg.draft), Wdn)
    ref = spec.target_only(ref_pair.target_rows, prompt, 24, scfg)
    assert res.tokens == ref
    assert len(res.tokens) == 12 + 24
    # with early stopping too
    pair2 = spec.TransformerPair(oshape(cfg.target), Wtn, oshape(cfg.draft), Wdn)
    c2 = gt.Controller(gt.Params(gamma_max=8), 4)
    res2 = spec.generate(pair2.draft_next, pair2.target_rows, prompt, 24, c2, spec.StepConfig(temperature=0.0, tau=0.007))
    assert res2.tokens == ref
    assert any(st.k < g for st, g in zip(res2.steps, res2.gammas))  # the early stop did trigger
    assert any(st.k == g for st, g in zip(res2.steps, res2.gammas))


def test_generate_bookkeeping():
    cfg = synth.pair("tiny")
    Wt, Wd = synth.make_pair_weights(cfg, 0)
    Wtn, Wdn = synth.to_numpy_weights(Wt), synth.to_numpy_weights(Wd)
    prompt = synth.make_prompts(1, 8, cfg.target.vocab, 9)[0].tolist()
    pairm = spec.TransformerPair(oshape(cfg.target), Wtn, oshape(cfg.draft), Wdn)
    c = gt.Controller(gt.Params(gamma_max=8), 4)
    res = spec.generate(pairm.draft_next, pairm.target_rows, prompt, 20, c, spec.StepConfig(temperature=1.0, seed=0))
    assert len(res.tokens) == 28 and res.tokens[:8] == prompt
    flat = [t for st in res.steps for t in st.emitted]
    assert flat[:20] == res.tokens[8:]
    for st, g in zip(res.steps, res.gammas):
        assert 1 <= st.k <= g and 0 <= st.accepted <= st.k and len(st.emitted) == st.accepted + 1
    # controller trajectory replays from the accept counts
    c2 = gt.Controller(gt.Params(gamma_max=8), 4)
    replay = [4]
    for st in res.steps:
        replay.append(c2.update(st.accepted, st.k))
    assert replay[:-1] == res.gammas


def test_pair_callables_equal_one_shot_forward_under_rollbacks():
    """TransformerPair keeps a cache per model and truncates it to the longest prefix it shares with the new token
    list, always leaving keep_back tokens (1 for the draft, k + 1 for the target) to feed.  Whatever the history of
    calls — growth, rejected suffixes rolled back, a list shorter than the cache, an unrelated list — every call must
    return what a cache-free forward of the full list returns (results are defined cache-free)."""
    cfg = synth.pair("tiny")
    Wt, Wd = synth.make_pair_weights(cfg, 3)
    Wtn, Wdn = synth.to_numpy_weights(Wt), synth.to_numpy_weights(Wd)
    st_, sd_ = oshape(cfg.target), oshape(cfg.draft)
    pairm = spec.TransformerPair(st_, Wtn, sd_, Wdn)
    base = synth.make_prompts(1, 14, cfg.target.vocab, 5)[0].tolist()
    other = synth.make_prompts(1, 14, cfg.target.vocab, 6)[0].tolist()
    histories = [
        base[:8],                       # first call: everything is fed
        base[:9], base[:10],            # growth by one token (draft passes of a step)
        base[:8] + other[8:11],         # rollback: last two rejected, three new ones
        base[:8] + other[8:9],          # shorter than the cache, same prefix
        base[:8] + other[8:9],          # identical list again: keep_back still re-feeds the tail
        other[:6],                      # unrelated list
        base[:14],
    ]
    for toks in histories:
        got = pairm.draft_next(toks)
        want = om.forward(sd_, Wdn, toks)[-1]
        assert np.max(np.abs(got - want)) < 1e-11
    for toks, k in [(base[:8], 0), (base[:12], 4), (base[:9] + other[9:12], 2), (base[:9] + other[9:12], 2),
                    (base[:6], 5), (other[:13], 1), (base[:14], 13)]:
        got = pairm.target_rows(toks, k)
        want = om.forward(st_, Wtn, toks)[-(k + 1):]
        assert got.shape == (k + 1, cfg.target.vocab)
        assert np.max(np.abs(got - want)) < 1e-11


def test_pair_sync_leaves_keep_back_tokens_to_feed():
    sh = oshape(synth.pair("tiny").target)
    cache = om.KVCache(sh)
    have = [1, 2, 3, 4, 5]
    # same list, keep_back 1: at most len - 1 positions may stay cached
    assert spec.TransformerPair._sync(cache, have, [1, 2, 3, 4, 5], 1) == 4
    # keep_back 3: two stay
    assert spec.TransformerPair._sync(cache, have, [1, 2, 3, 4, 5], 3) == 2
    # divergence at index 2 wins over keep_back
    assert spec.TransformerPair._sync(cache, have, [1, 2, 9, 4, 5, 6], 1) == 2
    # the new list is shorter than keep_back allows: nothing stays
    assert spec.TransformerPair._sync(cache, have, [1, 2], 3) == 0
    assert spec.TransformerPair._sync(cache, [], [1, 2, 3], 1) == 0
