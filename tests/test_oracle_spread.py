"""Pins of the oracle's spread of predicted order statistics (the bands of Fig. 3) — CPU only."""
import math

import numpy as np
import pytest

import oracle


def test_hand_worked_matrix_and_divisor():
    # rows sort to (1,2,5), (0,4,9), (2,3,4): rank means 1, 3, 6
    x = np.array([[5.0, 1.0, 2.0], [4.0, 9.0, 0.0], [2.0, 3.0, 4.0]])
    mean, sd = oracle.rank_spread(x)
    assert np.allclose(mean, [1.0, 3.0, 6.0], rtol=0, atol=1e-15)
    want = [math.sqrt((0 + 1 + 1) / 3), math.sqrt((1 + 1 + 0) / 3), math.sqrt((1 + 9 + 4) / 3)]
    assert np.allclose(sd, want, rtol=1e-15)
    # two rows: divisor S gives 1, the unbiased divisor S - 1 would give sqrt(2)
    _, sd2 = oracle.rank_spread(np.array([[0.0], [2.0]]))
    assert sd2[0] == 1.0


def test_uniform_order_statistics_are_beta():
    S, N = 60000, 7
    x = np.random.default_rng(1).random((S, N))
    mean, sd = oracle.rank_spread(x)
    c = np.arange(1, N + 1)
    assert np.allclose(mean, c / (N + 1), atol=4 * 0.2 / math.sqrt(S))
    want = np.sqrt(c * (N - c + 1) / ((N + 1) ** 2 * (N + 2)))
    assert np.allclose(sd, want, rtol=0.02)


def test_exponential_order_statistics_renyi():
    S, N = 60000, 6
    x = np.random.default_rng(2).exponential(size=(S, N))
    _, sd = oracle.rank_spread(x)
    want = np.sqrt([sum(1.0 / i ** 2 for i in range(N - c + 1, N + 1)) for c in range(1, N + 1)])
    assert np.allclose(sd, want, rtol=0.03)


def test_maximum_of_two_normals():
    x = np.random.default_rng(3).standard_normal((80000, 2))
    mean, sd = oracle.rank_spread(x)
    assert abs(mean[1] - 1 / math.sqrt(math.pi)) < 0.01 and abs(mean[0] + 1 / math.sqrt(math.pi)) < 0.01
    assert np.allclose(sd, math.sqrt(1 - 1 / math.pi), rtol=0.02)


def test_degenerate_and_affine_cases():
    g = np.random.default_rng(4)
    row = g.random(9)
    same = np.stack([g.permutation(row) for _ in range(20)])   # identical multisets, shuffled
    mean, sd = oracle.rank_spread(same)
    assert np.array_equal(mean, np.sort(row)) or np.allclose(mean, np.sort(row), rtol=1e-15)
    assert np.all(sd < 1e-15)
    x = g.random((500, 12))
    m1, s1 = oracle.rank_spread(x)
    m2, s2 = oracle.rank_spread(3.5 * x + 2.0)
    assert np.allclose(m2, 3.5 * m1 + 2.0, rtol=1e-13) and np.allclose(s2, 3.5 * s1, rtol=1e-12)
    # a decreasing map reverses the ranks
    m3, s3 = oracle.rank_spread(-x)
    assert np.allclose(m3, -m1[::-1], rtol=1e-13) and np.allclose(s3, s1[::-1], rtol=1e-12)
    # the means are the ones the cutoff rule uses
    assert np.allclose(m1, oracle.cutoff_select(x, want_sorted=False, want_perm=False)["mean"], rtol=1e-15)
    # one row: no spread
    _, s4 = oracle.rank_spread(x[:1])
    assert np.all(s4 == 0.0)


def test_bad_arguments():
    with pytest.raises(ValueError):
        oracle.rank_spread(np.zeros(5))
    with pytest.raises(ValueError):
        oracle.rank_spread(np.zeros((0, 5)))
