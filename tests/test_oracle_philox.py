"""Pins for oracle.philox: published known-answer vectors, scalar == vectorised, uniformity."""
import os

import numpy as np

from oracle import philox

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat():
    rows = []
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        w = [int(x, 16) for x in line.split()]
        rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_known_answers():
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, exp in rows:
        assert list(philox.philox4x32_10(ctr, key)) == exp


def test_array_matches_scalar():
    rng = np.random.default_rng(1)
    ctr = rng.integers(0, 2**32, size=(257, 4), dtype=np.uint64)
    key = (0x12345678, 0x9ABCDEF0)
    out = philox.philox4x32_10_array(ctr, key)
    for i in range(ctr.shape[0]):
        assert tuple(int(x) for x in out[i]) == philox.philox4x32_10(ctr[i], key)


def test_uniform_range_and_resolution():
    us = [philox.uniform(0, s, 1, philox.ACCEPT, 0) for s in range(2000)]
    assert min(us) >= 0.0 and max(us) < 1.0
    # 24-bit lattice: exactly representable in fp32
    for u in us[:100]:
        assert u * 16777216.0 == int(u * 16777216.0)
        assert np.float32(u) == u


def test_uniformity_chi_square():
    n = 200000
    ctr = np.zeros((n, 4), dtype=np.uint64)
    ctr[:, 0] = np.arange(n)
    ctr[:, 1] = 1
    ctr[:, 2] = philox.ACCEPT
    w0 = philox.philox4x32_10_array(ctr, philox.seed_key(0))[:, 0]
    u = (w0 >> 8).astype(np.float64) / 16777216.0
    hist, _ = np.histogram(u, bins=64, range=(0.0, 1.0))
    chi2 = ((hist - n / 64) ** 2 / (n / 64)).sum()
    assert chi2 < 120.0  # 63 dof: P(chi2 > 120) ~ 1e-5
    assert abs(u.mean() - 0.5) < 4 * (1 / 12 / n) ** 0.5


def test_streams_differ_by_purpose_row_sequence_and_seed():
    base = philox.uniform(7, 3, 2, philox.DRAFT, 0)
    others = [
        philox.uniform(7, 3, 2, philox.ACCEPT, 0),
        philox.uniform(7, 3, 3, philox.DRAFT, 0),
        philox.uniform(7, 4, 2, philox.DRAFT, 0),
        philox.uniform(7, 3, 2, philox.DRAFT, 1),
        philox.uniform(8, 3, 2, philox.DRAFT, 0),
        philox.uniform(7 + (1 << 32), 3, 2, philox.DRAFT, 0),
    ]
    assert all(o != base for o in others)
    assert philox.forced_uniform(7, 5, 0) == philox.uniform(7, 5, 0, philox.FORCED, 0)
