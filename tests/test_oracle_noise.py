"""Pins for the oracle's counter-based noise generator (CPU only)."""
import numpy as np
from scipy import stats

import oracle


def test_philox_known_answers(golden_dir):
    rows = [l.split() for l in (golden_dir / "philox4x32_10_kat.txt").read_text().splitlines()
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        assert oracle.philox4x32_10(w[0:4], w[4:6]) == w[6:10]


def test_normals_are_standard_and_streams_differ():
    a = oracle.fill_normal(12345, 0, (400000,)).astype(np.float64)
    assert abs(a.mean()) < 5 / np.sqrt(a.size) and abs(a.var() - 1) < 5 * np.sqrt(2 / a.size)
    assert abs(stats.skew(a)) < 0.02 and abs(stats.kurtosis(a)) < 0.04
    assert stats.kstest(a, "norm").pvalue > 1e-3
    lag1 = np.corrcoef(a[:-1], a[1:])[0, 1]
    assert abs(lag1) < 5 / np.sqrt(a.size)
    b = oracle.fill_normal(12345, 1, (1000,))
    c = oracle.fill_normal(12346, 0, (1000,))
    assert not np.array_equal(a[:1000].astype(np.float32), b) and not np.array_equal(a[:1000].astype(np.float32), c)
    # prefix property: element i does not depend on the tensor's length
    assert np.array_equal(oracle.fill_normal(7, 2, (10,)), oracle.fill_normal(7, 2, (1003,))[:10])
    # tail bound of the 24-bit uniform: |n| <= sqrt(2 * 24 * ln 2)
    assert np.abs(a).max() <= np.sqrt(2 * 24 * np.log(2)) + 1e-6
