"""The 8-bit weight generator: what the quantised model is (q, scale) and what the oracle is handed for it."""
import numpy as np
import torch

import synth


def test_quantize_rows_bounds_and_error():
    g = torch.Generator().manual_seed(3)
    w = torch.randn(37, 200, generator=g) * 0.02
    w[5] = 0.0  # an all-zero row must not divide by zero
    q, s = synth.quantize_rows(w)
    assert q.dtype == torch.int8 and s.dtype == torch.float32 and q.shape == w.shape and s.shape == (37,)
    assert int(q.abs().max()) <= 127
    nz = [r for r in range(37) if r != 5]
    np.testing.assert_allclose(s[nz].numpy(), (w[nz].abs().amax(dim=1) / 127.0).numpy(), rtol=1e-6)
    # every row reaches +-127 somewhere, and rounding to the nearest step leaves at most half a step
    assert (q[nz].abs().amax(dim=1) == 127).all()
    err = (w - s[:, None] * q.float()).abs()
    assert (err <= 0.5 * s[:, None] * (1 + 1e-5) + 1e-12).all()
    assert (q[5] == 0).all()


def test_oracle_receives_scale_times_q():
    cfg = synth.pair("small-q8")
    Wt, Wd = synth.make_pair_weights(cfg, 0)
    n = synth.to_numpy_weights(Wt)
    assert not any(k.endswith("_scale") for k in n)
    for k in ("wq", "w_down"):
        q, s = Wt[k][1], Wt[k + "_scale"][1]
        assert n[k][1].dtype == np.float64
        np.testing.assert_array_equal(n[k][1], s.double().numpy()[:, None] * q.double().numpy())
    np.testing.assert_array_equal(n["lm_head"], Wt["lm_head_scale"].double().numpy()[:, None] * Wt["lm_head"].double().numpy())
    assert n["tok_embed"].dtype == np.uint16 and n["final_norm"].dtype == np.uint16  # bf16 bit patterns, untouched
