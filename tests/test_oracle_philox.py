"""Pins for oracle/philox.py: published known-answer vectors and basic statistics."""
import os

import numpy as np

from oracle.philox import philox4x32_10, uniform_for

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_known_answer_vectors():
    rows = [l.split() for l in open(GOLD) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        assert philox4x32_10(w[0:4], w[4:6]) == tuple(w[6:10])


def test_uniform_range_and_moments():
    u = np.array([uniform_for(7, rid, g) for rid in range(40) for g in range(100)])
    assert u.min() >= 0.0 and u.max() < 1.0
    # 4000 uniforms: mean 0.5 +- 5 sigma, variance 1/12
    assert abs(u.mean() - 0.5) < 5 * (1 / 12 / 4000) ** 0.5
    assert abs(u.var() - 1 / 12) < 0.01
    # 24-bit grid
    assert np.all(u * 2 ** 24 == np.floor(u * 2 ** 24))


def test_streams_are_keyed_by_request_and_index():
    a = uniform_for(1, 5, 9)
    assert a == uniform_for(1, 5, 9)
    assert a != uniform_for(2, 5, 9) and a != uniform_for(1, 6, 9) and a != uniform_for(1, 5, 10)
    # 64-bit request ids use the high counter word
    assert uniform_for(1, 5 + (1 << 32), 9) != a
