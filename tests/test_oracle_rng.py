"""Pins for the oracle's counter-based uniforms (reading: Philox-4x32-10, 23-bit grid of odd multiples of 2^-24)."""
import os

import numpy as np

from oracle import s2d2_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_philox_known_answers():
    n = 0
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(x, 16) for x in line.split()]
        assert list(O.philox4x32_10(v[:4], v[4:6])) == v[6:]
        n += 1
    assert n >= 2


def test_uniform_open_interval_and_fp32_exact():
    us = np.array([O.uniform(7, s, n, i, st) for s in range(4) for n in range(4) for i in range(8) for st in range(3)])
    assert (us > 0).all() and (us < 1).all()
    assert (us.astype(np.float32).astype(np.float64) == us).all()  # exactly representable in fp32
    assert len(np.unique(us)) > 0.99 * len(us)
    assert abs(us.mean() - 0.5) < 0.06


def test_uniform_depends_on_every_counter_word_and_key():
    base = O.uniform(1, 2, 3, 4, 0)
    others = [O.uniform(2, 2, 3, 4, 0), O.uniform(1, 3, 3, 4, 0), O.uniform(1, 2, 4, 4, 0),
              O.uniform(1, 2, 3, 5, 0), O.uniform(1, 2, 3, 4, 1), O.uniform(1 + (1 << 32), 2, 3, 4, 0)]
    assert all(o != base for o in others)


def test_uniform_grid_statistics():
    # 23-bit grid: u * 2^23 - 0.5 is an integer in [0, 2^23)
    us = np.array([O.uniform(0, 0, 0, i, 0) for i in range(2000)])
    k = us * 8388608.0 - 0.5
    assert (k == np.round(k)).all() and k.min() >= 0 and k.max() < 8388608
    hist, _ = np.histogram(us, bins=10, range=(0, 1))
    assert hist.min() > 140 and hist.max() < 260
