"""Pins for the oracle's random numbers (the "with probability p_r" of Eq. (2))."""
import os

import numpy as np

from oracle import binding as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _vectors():
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        w = [int(t, 16) for t in line.split()]
        yield w[0:4], w[4:6], w[6:10]


def test_philox_known_answers():
    n = 0
    for ctr, key, want in _vectors():
        got = O.philox4x32(ctr, key, 10)
        assert [int(x) for x in got] == want
        n += 1
    assert n == 3


def test_philox_is_a_bijection_of_the_counter_sample():
    # a keyed permutation of the 128-bit counter: distinct counters, distinct outputs
    seen = set()
    for c in range(2000):
        seen.add(tuple(int(x) for x in O.philox4x32([c, 0, 7, 9], [123, 456], 10)))
    assert len(seen) == 2000


def test_rand16_takes_the_stated_halves_of_the_stated_words():
    seed, worker, step = 0x0123456789ABCDEF, 5, 77
    for e in [0, 1, 7, 8, 13, 8 * 12345 + 6, (1 << 35) + 3]:
        q = e >> 3
        w = O.philox4x32([q & 0xFFFFFFFF, q >> 32, worker, step],
                         [seed & 0xFFFFFFFF, seed >> 32], 10)
        j = e & 7
        want = (int(w[j >> 1]) >> (16 * (j & 1))) & 0xFFFF
        assert O.rand16(seed, worker, step, e) == want


def test_rand16_is_uniform_and_decorrelated():
    # chi-square of the top 4 bits over 64k consecutive elements; neighbours uncorrelated
    r = np.array([O.rand16(42, 1, 3, e) for e in range(1 << 16)], dtype=np.float64)
    counts = np.bincount((r.astype(np.int64) >> 12), minlength=16)
    expect = r.size / 16
    chi2 = ((counts - expect) ** 2 / expect).sum()
    assert chi2 < 45.0            # 15 dof, p ~ 1e-4
    u = r / 65536.0
    assert abs(u.mean() - 0.5) < 4 * (1 / 12) ** 0.5 / r.size ** 0.5 + 1e-5
    c = np.corrcoef(u[:-1], u[1:])[0, 1]
    assert abs(c) < 4 / r.size ** 0.5
    # other worker / other step: different streams
    r2 = np.array([O.rand16(42, 2, 3, e) for e in range(4096)])
    r3 = np.array([O.rand16(42, 1, 4, e) for e in range(4096)])
    assert (r2 != r[:4096]).mean() > 0.99 and (r3 != r[:4096]).mean() > 0.99
