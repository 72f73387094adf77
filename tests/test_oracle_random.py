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
    big = oracle.random_normal(7, (1 << 34) - 5, 10, 1.0)                          # the counter crosses 2^32
    assert np.array_equal(big[5:], oracle.random_normal(7, 1 << 34, 5, 1.0))
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


def test_four_stream_positions_share_one_generator_call():
    """Positions 4c..4c+3 come from the four words of counter c: words (0,1) give the cosine and the sine of
    one Box-Muller pair, words (2,3) those of the other."""
    c = 5
    w = [int(x) for x in oracle.philox4x32_10([c, 0, 0, 0], [9, 0])]
    u = [((x >> 8) + 0.5) / 2 ** 24 for x in w]
    z = oracle.random_normal(9, 4 * c, 4, 1.0)
    want = [np.sqrt(-2 * np.log(u[0])) * np.cos(2 * np.pi * u[1]), np.sqrt(-2 * np.log(u[0])) * np.sin(2 * np.pi * u[1]),
            np.sqrt(-2 * np.log(u[2])) * np.cos(2 * np.pi * u[3]), np.sqrt(-2 * np.log(u[2])) * np.sin(2 * np.pi * u[3])]
    assert np.allclose(z, want, rtol=1e-12)
    # the two values of a pair lie on one circle of radius sqrt(-2 ln u1)
    assert np.isclose(z[0] ** 2 + z[1] ** 2, -2 * np.log(u[0]), rtol=1e-12)
    # a counter beyond 2^32 uses the high counter word
    hi = oracle.random_normal(9, (1 << 34) + 4, 1, 1.0)[0]
    wh = [int(x) for x in oracle.philox4x32_10([1, 1, 0, 0], [9, 0])]
    uh = [((x >> 8) + 0.5) / 2 ** 24 for x in wh]
    assert np.isclose(hi, np.sqrt(-2 * np.log(uh[0])) * np.cos(2 * np.pi * uh[1]), rtol=1e-12)


def test_values_of_one_call_are_uncorrelated():
    n = 400_000
    z = oracle.random_normal(3, 0, n, 1.0).reshape(-1, 4)
    corr = np.corrcoef(z.T)
    assert np.abs(corr - np.eye(4)).max() < 5 / np.sqrt(n / 4)
    # and so are their squares (cosine and sine of one angle are uncorrelated but share a radius only in magnitude)
    corr2 = np.corrcoef((z ** 2).T)
    assert np.abs(corr2 - np.eye(4)).max() < 6 / np.sqrt(n / 4)
