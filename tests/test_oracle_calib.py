"""Pins of the oracle's offline calibration (CPU only): Section 5.1 of the paper picks the
outlier channels by the highest square sum over calibration activations and reorders by them."""
from fractions import Fraction

import numpy as np

import oracle


def test_exact_small_integers():
    """Activations that are small integers: every square sum is an exact integer whatever the
    order of the additions, so numpy's int64 arithmetic pins statistic and index."""
    rng = np.random.default_rng(0)
    x = rng.integers(-8, 9, (700, 96)).astype(np.float16)
    x[:, 5] = x[:, 17]                                  # two equal channels keep their order
    stat, idx = oracle.calibrate_reorder(x)
    want = (x.astype(np.int64) ** 2).sum(axis=0)
    assert np.array_equal(stat, want.astype(np.float64))
    order = sorted(range(96), key=lambda k: (int(want[k]), k))
    assert idx.tolist() == order
    assert idx.tolist().index(5) + 1 == idx.tolist().index(17)


def test_statistic_against_exact_rationals_and_numpy():
    rng = np.random.default_rng(1)
    sigma = np.exp(1.5 * rng.standard_normal(64))
    x = (rng.standard_normal((1000, 64)) * sigma).astype(np.float16)
    stat, idx = oracle.calibrate_reorder(x)
    for k in (0, 13, 63):
        exact = sum(Fraction(float(v)) ** 2 for v in x[:, k])
        assert abs(Fraction(float(stat[k])) - exact) <= exact * Fraction(1, 2 ** 45)
    ref = np.square(x.astype(np.float64)).sum(axis=0)
    assert np.allclose(stat, ref, rtol=1e-12, atol=0)
    # heavy-tailed channels are far apart: the index is the plain stable argsort
    assert np.array_equal(idx, np.argsort(ref, kind="stable").astype(np.int32))
    # a permutation whose last 8 entries are the 8 largest channels
    assert sorted(idx.tolist()) == list(range(64))
    assert set(idx[-8:].tolist()) == set(np.argsort(ref)[-8:].tolist())


def test_chunking_and_edge_shapes():
    x = np.ones((513, 4), np.float16)                   # 2 full chunks and one row
    x[:, 1] = 2
    x[:, 2] = 0
    stat, idx = oracle.calibrate_reorder(x)
    assert stat.tolist() == [513.0, 2052.0, 0.0, 513.0]
    assert idx.tolist() == [2, 0, 3, 1]
    stat, idx = oracle.calibrate_reorder(np.zeros((0, 8), np.float16))
    assert not stat.any() and idx.tolist() == list(range(8))
