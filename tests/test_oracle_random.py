"""Pins for the oracle's random-gradient stream (CPU only): the published
known-answer vectors of Philox4x32-10, and the distribution the method asks for
(Section 2.2: independent N(0, sigma), fresh numbers for every batch)."""
import os

import numpy as np
import scipy.stats

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_philox_known_answers():
    rows = [l for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for row in rows:
        ctr, key, out = [[int(x, 16) for x in part.split()] for part in row.split("|")]
        assert oracle.philox4x32_10(ctr, key).tolist() == out


def test_stream_is_a_pure_function_of_seed_and_global_index():
    a = oracle.random_normal(7, 0, 1000, 1 / 128)
    assert np.array_equal(a, oracle.random_normal(7, 0, 1000, 1 / 128))
    assert np.array_equal(a[300:], oracle.random_normal(7, 300, 700, 1 / 128))   # offset = position
    assert not np.array_equal(a, oracle.random_normal(8, 0, 1000, 1 / 128))
    big = oracle.random_normal(7, (1 << 32) - 5, 10, 1.0)                          # crosses 2^32
    assert np.array_equal(big[5:], oracle.random_normal(7, 1 << 32, 5, 1.0))
    assert np.array_equal(oracle.random_normal(7, 0, 10, 0.5), 64 * oracle.random_normal(7, 0, 10, 1 / 128))


def test_distribution_is_standard_normal_times_sigma():
    n, sigma = 400_000, 1 / 128
    z = oracle.random_normal(190805460, 12345, n, sigma) / sigma
    assert abs(z.mean()) < 4 / np.sqrt(n)
    assert abs(z.std() - 1) < 0.01
    assert scipy.stats.kstest(z, "norm").pvalue > 1e-3
    assert abs(scipy.stats.skew(z)) < 0.02 and abs(scipy.stats.kurtosis(z)) < 0.05
    assert abs(np.corrcoef(z[:-1], z[1:])[0, 1]) < 4 / np.sqrt(n)                # lag-1
    assert np.abs(z).max() < np.sqrt(2 * np.log(2.0 ** 25)) + 1e-9              # Box-Muller's range


def test_box_muller_uses_the_first_two_words():
    """u1 from word 0 sets the radius, u2 from word 1 the angle: recover both from a
    sample pair generated with the cosine (here) and check the radius bound."""
    w = oracle.philox4x32_10([5, 0, 0, 0], [9, 0])
    u1 = ((int(w[0]) >> 8) + 0.5) / 2 ** 24
    u2 = ((int(w[1]) >> 8) + 0.5) / 2 ** 24
    z = oracle.random_normal(9, 5, 1, 1.0)[0]
    assert np.isclose(z, np.sqrt(-2 * np.log(u1)) * np.cos(2 * np.pi * u2), rtol=1e-12)
