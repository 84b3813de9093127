"""Pins of the oracle's counter-based generator.  CPU only."""
import os

import numpy as np

from oracle.philox import philox4x32_10, uniform24

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_known_answers():
    n = 0
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(t, 16) for t in line.split()]
        assert list(philox4x32_10(tuple(v[0:4]), tuple(v[4:6]))) == v[6:10]
        n += 1
    assert n == 3


def test_uniform_grid_range_and_moments():
    us = np.array([uniform24(1234, 0, s, k) for s in range(400) for k in range(5)])
    assert us.min() >= 0.0 and us.max() < 1.0
    assert np.all(us * (1 << 24) == np.floor(us * (1 << 24)))          # on the 2^-24 grid
    assert np.all(us.astype(np.float32).astype(np.float64) == us)      # exactly representable in fp32
    assert abs(us.mean() - 0.5) < 0.03 and abs(us.var() - 1 / 12) < 0.01
    hist = np.histogram(us, bins=10, range=(0, 1))[0]
    assert ((hist - 200.0) ** 2 / 200.0).sum() < 30.0                  # chi-square, 9 dof


def test_streams_differ_by_every_counter_field():
    base = uniform24(7, 1, 2, 3)
    assert len({base, uniform24(8, 1, 2, 3), uniform24(7, 2, 2, 3), uniform24(7, 1, 3, 3), uniform24(7, 1, 2, 4),
                uniform24(7 + (1 << 32), 1, 2, 3), uniform24(7, 1, 2 + (1 << 32), 3)}) == 7
