"""Pins for the oracle's counter-based generator (Philox4x32-10) and its use.

What fixes it from outside: the published known-answer vectors, the stated
counter/key layout (checked by re-deriving the accept uniform and the Gumbel
noise from raw Philox words), and distributional tests.
"""
import math
import os

import numpy as np
import pytest
from scipy import stats

import oracle

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


def test_known_answer_vectors():
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, want in rows:
        got = oracle.philox4x32_10(ctr, key)
        assert [int(x) for x in got] == want


def test_counter_is_sensitive_to_every_word():
    base = oracle.philox4x32_10([1, 2, 3, 4], [5, 6])
    for pos in range(4):
        c = [1, 2, 3, 4]
        c[pos] ^= 1
        assert not np.array_equal(oracle.philox4x32_10(c, [5, 6]), base)
    for pos in range(2):
        k = [5, 6]
        k[pos] ^= 1
        assert not np.array_equal(oracle.philox4x32_10([1, 2, 3, 4], k), base)


def _u(word):
    return (2 * (int(word) >> 9) + 1) / 2.0 ** 24


def test_accept_uniform_layout():
    """u of logit row `row` = word 0 of counter (0,row,0,offset), key = (seed lo, seed hi)."""
    seed = 0x0123456789ABCDEF
    for row, off in [(0, 0), (5, 0), (77, 3), (4095, 1234567)]:
        w = oracle.philox4x32_10([0, row, 0, off], [seed & 0xFFFFFFFF, seed >> 32])
        assert oracle.accept_uniform(seed, off, row) == _u(w[0])


def test_gumbel_layout():
    """Noise of element i of row `row` = word i&3 of counter (i>>2,row,1,offset)."""
    seed = 0xFEDCBA9876543210
    for row, off, i in [(0, 0, 0), (3, 0, 1), (3, 9, 2), (8, 1, 3), (8, 1, 4), (100, 7, 151935)]:
        w = oracle.philox4x32_10([i >> 2, row, 1, off], [seed & 0xFFFFFFFF, seed >> 32])
        u = _u(w[i & 3])
        assert oracle.gumbel(seed, off, row, i) == pytest.approx(-math.log(-math.log(u)), rel=1e-14)


def test_uniform_is_exact_fp32_and_open_interval():
    assert _u(0) == 2.0 ** -24 and _u(0xFFFFFFFF) == 1 - 2.0 ** -24
    us = np.array([oracle.accept_uniform(42, 0, r) for r in range(20000)])
    assert us.min() > 0.0 and us.max() < 1.0
    assert np.array_equal(us.astype(np.float32).astype(np.float64), us)  # exact in fp32
    # Kolmogorov-Smirnov against U(0,1)
    assert stats.kstest(us, "uniform").pvalue > 1e-3
    assert abs(us.mean() - 0.5) < 0.01 and abs(us.var() - 1 / 12) < 0.005


def test_gumbel_moments():
    g = np.array([oracle.gumbel(7, 0, 11, i) for i in range(40000)])
    assert abs(g.mean() - 0.5772156649) < 0.03          # Euler-Mascheroni
    assert abs(g.var() - math.pi ** 2 / 6) < 0.06
    assert stats.kstest(g, "gumbel_r").pvalue > 1e-3


def test_streams_and_rows_are_independent():
    a = np.array([oracle.gumbel(1, 0, 0, i) for i in range(4000)])
    b = np.array([oracle.gumbel(1, 0, 1, i) for i in range(4000)])
    c = np.array([oracle.gumbel(1, 1, 0, i) for i in range(4000)])
    assert abs(np.corrcoef(a, b)[0, 1]) < 0.06
    assert abs(np.corrcoef(a, c)[0, 1]) < 0.06


def test_batched_dump_is_the_scalar_functions_element_by_element():
    u, g = oracle.rng_dump(99, 3, 1, 17, 2, 37)
    for r in range(2):
        for i in (0, 1, 2, 3, 4, 35, 36):
            assert g[r, i] == oracle.gumbel(99, 3, 17 + r, i)
            word = oracle.philox4x32_10([i >> 2, 17 + r, 1, 3], [99, 0])[i & 3]
            assert u[r, i] == (2 * (int(word) >> 9) + 1) * 2.0 ** -24
    u0, _ = oracle.rng_dump(99, 3, 0, 17, 2, 4)
    assert u0[1, 0] == oracle.accept_uniform(99, 3, 18)
