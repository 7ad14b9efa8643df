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
    # the statistic is the exact rational sum rounded once (Fraction -> float rounds to nearest even)
    for k in range(64):
        exact = sum(Fraction(float(v)) ** 2 for v in x[:, k])
        assert float(stat[k]) == float(exact)
    # ... which no fixed order of double additions reproduces on every channel of this input: a
    # chunked or a sequential double sum in place of the exact one fails this pin
    x64 = x.astype(np.float64) ** 2
    seq = np.zeros(64)
    for t in range(1000):
        seq += x64[t]
    chunk = sum(x64[c:c + 256].sum(axis=0) for c in range(0, 1000, 256))
    assert (seq != stat).any() and (chunk != stat).any()
    ref = np.square(x.astype(np.float64)).sum(axis=0)
    assert np.allclose(stat, ref, rtol=1e-12, atol=0)
    # heavy-tailed channels are far apart: the index is the plain stable argsort
    assert np.array_equal(idx, np.argsort(ref, kind="stable").astype(np.int32))
    # a permutation whose last 8 entries are the 8 largest channels
    assert sorted(idx.tolist()) == list(range(64))
    assert set(idx[-8:].tolist()) == set(np.argsort(ref)[-8:].tolist())


def test_order_of_rows_does_not_matter_and_special_values():
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((900, 32)) * np.exp(2.0 * rng.standard_normal(32))).astype(np.float16)
    x[::2, 0] = 65504.0
    x[1::2, 0] = 6e-8                                     # the smallest subnormal beside the largest value
    x[:, 1] = 6e-8
    stat, idx = oracle.calibrate_reorder(x)
    s2, i2 = oracle.calibrate_reorder(x[rng.permutation(900)])
    assert np.array_equal(stat.view(np.uint64), s2.view(np.uint64)) and np.array_equal(idx, i2)
    tiny = float(np.float16(6e-8)) ** 2
    assert stat[1] == 900 * tiny                          # 900 * 2^-48: exact
    assert stat[0] == float(450 * Fraction(65504) ** 2 + 450 * Fraction(tiny))
    y = np.ones((4, 3), np.float16)
    y[0, 1] = np.inf
    y[1, 2] = np.nan
    stat, idx = oracle.calibrate_reorder(y)               # Inf and NaN count as magnitude 2^16
    assert stat.tolist() == [4.0, 3.0 + 2.0 ** 32, 3.0 + 2.0 ** 32] and idx.tolist() == [0, 1, 2]


def test_chunking_and_edge_shapes():
    x = np.ones((513, 4), np.float16)                   # 2 full chunks and one row
    x[:, 1] = 2
    x[:, 2] = 0
    stat, idx = oracle.calibrate_reorder(x)
    assert stat.tolist() == [513.0, 2052.0, 0.0, 513.0]
    assert idx.tolist() == [2, 0, 3, 1]
    stat, idx = oracle.calibrate_reorder(np.zeros((0, 8), np.float16))
    assert not stat.any() and idx.tolist() == list(range(8))
