"""Pins of the oracle's Philox4x32-10 and of its uniform / normal transforms (no GPU)."""
import os

import numpy as np
from scipy import stats

from oracle import philox

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_known_answer_vectors():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(h, 16) for h in r]
        out = philox.philox4x32_10(np.array(v[0:4], np.uint32), np.array(v[4:6], np.uint32))
        assert [int(o) for o in out] == v[6:10]


def test_counter_fields_are_independent_streams():
    base = philox.normal(5, [3], [7], 8)
    assert not np.allclose(base, philox.normal(5, [4], [7], 8))      # env changes the stream
    assert not np.allclose(base, philox.normal(5, [3], [8], 8))      # t changes the stream
    assert not np.allclose(base, philox.normal(6, [3], [7], 8))      # seed changes the stream
    assert not np.allclose(base, philox.normal(5 + (1 << 32), [3], [7], 8))  # high key word is used
    np.testing.assert_array_equal(base, philox.normal(5, [3], [7], 8))
    # a longer vector extends a shorter one (element e lives in block e // 4)
    np.testing.assert_array_equal(philox.normal(5, [3], [7], 10)[:, :8], base)
    # batch composition does not matter
    both = philox.normal(5, [9, 3], [1, 7], 8)
    np.testing.assert_array_equal(both[1:], base)


def test_uniform_range_and_law():
    n = 200_000
    u = philox.uniform(1, np.arange(n) % 1000, np.arange(n) // 1000)
    assert u.min() > 0 and u.max() < 1
    assert np.all(u.astype(np.float32).astype(np.float64) == u)       # exact in fp32
    assert stats.kstest(u, "uniform").pvalue > 1e-3
    assert abs(u.mean() - 0.5) < 4 / np.sqrt(12 * n)


def test_normal_law():
    z = philox.normal(2, np.arange(2000), np.full(2000, 17), 160).ravel()
    n = z.size
    assert stats.kstest(z, "norm").pvalue > 1e-3
    assert abs(z.mean()) < 4 / np.sqrt(n)
    assert abs(z.var() - 1) < 4 * np.sqrt(2 / n)
    assert abs(stats.kurtosis(z)) < 0.05
    # neighbouring elements (the cos / sin pair and the two pairs of a block) are uncorrelated
    zz = z.reshape(-1, 4)
    c = np.corrcoef(zz.T)
    assert np.abs(c - np.eye(4)).max() < 4 / np.sqrt(zz.shape[0])
