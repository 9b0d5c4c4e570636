"""Pins for oracle/philox.py: the generator's published known-answer vectors and
a uniformity chi-square (nothing here re-types the generator)."""
import os

import numpy as np
from scipy import stats

from oracle import philox

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox_kat.txt")


def _vectors():
    for line in open(GOLD):
        line = line.split("#")[0].split()
        if len(line) == 10:
            w = [int(t, 16) for t in line]
            yield w[:4], w[4:6], w[6:]


def test_known_answer_vectors():
    n = 0
    for ctr, key, out in _vectors():
        assert list(philox.philox4x32_10(ctr, key)) == out
        vec = philox.philox4x32_10_np(*ctr, *key)
        assert [int(v) for v in vec] == out
        n += 1
    assert n == 3


def test_uniform_is_24_bit_and_in_range():
    for slot in range(1, 50):
        u = philox.uniform(7, slot, 3, 0, 1)
        assert 0.0 <= u < 1.0
        assert u * 2 ** 24 == int(u * 2 ** 24)
        assert float(np.float32(u)) == u          # same real number in fp32 and fp64


def test_vectorised_equals_scalar():
    seeds = [0, 1, 2 ** 40 + 5]
    for seed in seeds:
        us = philox.uniform_np(seed, np.arange(1, 20), 5, 2, 1)
        for i, u in enumerate(us):
            assert u == philox.uniform(seed, i + 1, 5, 2, 1)


def test_uniformity_chi_square():
    u = philox.uniform_np(12345, np.arange(1, 200001), 0, 0, 0)
    counts = np.bincount((u * 64).astype(int), minlength=64)
    assert stats.chisquare(counts).pvalue > 1e-3
    # consecutive slots are not correlated (lag-1 pairs over a 8x8 grid)
    pair = (u[:-1] * 8).astype(int) * 8 + (u[1:] * 8).astype(int)
    assert stats.chisquare(np.bincount(pair, minlength=64)).pvalue > 1e-3


def test_streams_rounds_and_sequences_are_distinct():
    base = philox.uniform(9, 1, 0, 0, 0)
    others = [philox.uniform(9, 2, 0, 0, 0), philox.uniform(9, 1, 1, 0, 0),
              philox.uniform(9, 1, 0, 1, 0), philox.uniform(9, 1, 0, 0, 1), philox.uniform(10, 1, 0, 0, 0)]
    assert all(o != base for o in others)
