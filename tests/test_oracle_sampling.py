"""Pins of the oracle's stochastic sampling (Alg. 1 samples the output distribution): the counter-based generator
against its published known answers, the sampler against the distribution it is defined to draw from."""
import os

import numpy as np
import pytest

from oracle import mdi_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_known_answers.txt")


def test_philox_known_answers():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        assert list(O.philox4x32_10(v[0:4], v[4:6])) == v[6:10]


def test_philox_is_a_bijection_of_the_counter_on_a_small_slice():
    # distinct counters give distinct outputs (it is a keyed permutation); the key changes all of them
    a = {O.philox4x32_10((i, j, 0, 0), (1, 2)) for i in range(40) for j in range(40)}
    b = {O.philox4x32_10((i, j, 0, 0), (1, 3)) for i in range(40) for j in range(40)}
    assert len(a) == 1600 and len(b) == 1600 and not (a & b)


def test_uniform01_range_resolution_and_moments():
    u = np.array([O.uniform01(12345, s, t) for s in range(8) for t in range(2500)])
    assert u.min() >= 0.0 and u.max() < 1.0
    assert np.all(u * (1 << 24) == np.floor(u * (1 << 24)))            # 24-bit fractions: exact in binary32
    assert abs(u.mean() - 0.5) < 0.01 and abs(u.var() - 1 / 12) < 0.005
    hist = np.histogram(u, bins=20, range=(0, 1))[0]
    assert hist.min() > 850 and hist.max() < 1150                      # 1000 expected per bin
    assert O.uniform01(1, 2, 3) != O.uniform01(1, 3, 2) != O.uniform01(2, 2, 3)


def test_topk_of_one_is_greedy_and_ties_go_to_the_lower_index():
    rng = np.random.default_rng(0)
    lg = rng.standard_normal(50)
    for u in (0.0, 0.3, 0.999999):
        assert O.sample_topk(lg, 0.7, 1, u) == int(np.argmax(lg)) == O.greedy(lg)
    lg[7] = lg[31] = lg.max() + 1.0
    assert O.sample_topk(lg, 1.0, 1, 0.9) == 7
    assert O.sample_topk(lg, 1.0, 2, 0.49) == 7 and O.sample_topk(lg, 1.0, 2, 0.51) == 31


def test_inverse_cdf_intervals_have_the_lengths_of_the_pmf():
    """Brute force: sweep u over a fine grid; the share of the grid that maps to a token is its probability."""
    lg = np.array([2.0, -1.0, 0.5, 2.0, 1.25, -3.0, 0.0])
    for temperature, k in ((1.0, 7), (0.5, 4), (3.0, 5)):
        pmf = O.topk_pmf(lg, temperature, k)
        assert abs(sum(pmf.values()) - 1.0) < 1e-12 and len(pmf) == k
        n = 20000
        counts = {}
        for j in range(n):
            t = O.sample_topk(lg, temperature, k, (j + 0.5) / n)
            counts[t] = counts.get(t, 0) + 1
        assert set(counts) == set(pmf)
        for t, p in pmf.items():
            assert abs(counts[t] / n - p) < 2.0 / n + 1e-6, (temperature, k, t)
    # by hand: two candidates with logits 0 and ln 3 at temperature 1 -> probabilities 1/4 and 3/4
    two = np.array([0.0, np.log(3.0)])
    assert O.sample_topk(two, 1.0, 2, 0.74) == 1 and O.sample_topk(two, 1.0, 2, 0.76) == 0


def test_shift_invariance_temperature_limits_and_end_points():
    rng = np.random.default_rng(3)
    lg = rng.standard_normal(30) * 2
    for u in np.linspace(0.01, 0.99, 23):
        assert O.sample_topk(lg, 0.8, 10, u) == O.sample_topk(lg + 5.0, 0.8, 10, u)
        assert O.sample_topk(lg, 1e-3, 10, u) == int(np.argmax(lg))      # cold: the mass sits on the maximum
    order = np.argsort(-lg)
    assert O.sample_topk(lg, 1.0, 10, 0.0) == order[0]
    assert O.sample_topk(lg, 1.0, 10, 1.0 - 2.0 ** -24) == order[9]
    hot = O.topk_pmf(lg, 1e6, 10)                                        # hot: uniform over the top k
    assert max(hot.values()) - min(hot.values()) < 1e-4


def test_draws_follow_the_pmf():
    lg = np.array([1.0, 0.0, -0.5, 2.0, 1.5, 0.3])
    pmf = O.topk_pmf(lg, 0.9, 4)
    n = 12000
    counts = {}
    for step in range(n):
        t = O.sample_topk(lg, 0.9, 4, O.uniform01(99, 0, step))
        counts[t] = counts.get(t, 0) + 1
    chi2 = sum((counts.get(t, 0) - n * p) ** 2 / (n * p) for t, p in pmf.items())
    assert set(counts) <= set(pmf) and chi2 < 16.3                       # 3 degrees of freedom, p = 0.001
