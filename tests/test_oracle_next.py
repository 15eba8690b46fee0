"""Pins for the oracle's censored-run-time imputation (Sec. 4.2) and for the
comparison cutoffs (Elfving "order" baseline of eq. 4 / Sec. 4.1, full
synchronisation, hindsight maximum of Fig. 2).  CPU only.

Nothing here compares the oracle with itself: the truncated predictive is
checked against closed-form truncated means of known distributions, the
Elfving formula against the value the paper prints and against quadrature of
the exact order-statistic integral, the cutoffs against enumeration.
"""
import math
from pathlib import Path

import numpy as np
import pytest
from scipy import integrate, stats

import oracle

GOLDEN = Path(__file__).parent / "golden" / "paper_worked_examples.txt"


def read_golden():
    out = {}
    for line in GOLDEN.read_text().splitlines():
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = float(v)
    return out


# ---- censored run-times -------------------------------------------------------

def test_observed_workers_keep_their_times_and_dropped_ones_exceed_tau():
    rng = np.random.default_rng(5)
    S, N = 300, 40
    x = rng.lognormal(0.0, 0.3, size=(S, N)).astype(np.float32)
    obs = rng.lognormal(0.0, 0.3, size=N).astype(np.float32)
    cens = (rng.random(N) < 0.4).astype(np.uint8)
    tau = np.float32(1.1)
    u = rng.random(N).astype(np.float32)
    full, cnt = oracle.impute_censored(x, obs, cens, tau, u)
    keep = cens == 0
    assert np.array_equal(full[keep], obs[keep]) and np.all(cnt[keep] == -1)
    for w in np.flatnonzero(cens):
        assert cnt[w] == int(np.sum(x[:, w] > tau))
        assert full[w] > tau
        assert full[w] in x[:, w]          # one of that worker's own predictive draws


def test_pick_walks_through_the_exceeding_draws_in_sample_order():
    # one worker, draws 1..10, tau = 4.5 -> exceeding draws 5,6,7,8,9,10 in this order
    x = np.arange(1, 11, dtype=np.float32).reshape(10, 1)
    for i, expect in enumerate([5, 6, 7, 8, 9, 10]):
        u = np.array([(i + 0.5) / 6], dtype=np.float32)
        full, cnt = oracle.impute_censored(x, np.zeros(1, np.float32), np.ones(1, np.uint8), 4.5, u)
        assert cnt[0] == 6 and full[0] == expect
    # draws equal to tau do not exceed it (strict truncation: the worker was still running at tau)
    full, cnt = oracle.impute_censored(x, np.zeros(1, np.float32), np.ones(1, np.uint8), 5.0, np.zeros(1, np.float32))
    assert cnt[0] == 5 and full[0] == 6


def test_no_exceeding_draw_gives_tau():
    x = np.full((8, 3), 0.5, dtype=np.float32)
    full, cnt = oracle.impute_censored(x, np.ones(3, np.float32), np.array([1, 0, 1], np.uint8), 2.0,
                                       np.array([0.3, 0.3, 0.99], np.float32))
    assert full.tolist() == [2.0, 1.0, 2.0] and cnt.tolist() == [0, -1, 0]


def test_u_outside_unit_interval_is_rejected():
    x = np.ones((4, 1), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.impute_censored(x, np.ones(1, np.float32), np.ones(1, np.uint8), 0.5, np.array([1.0], np.float32))


@pytest.mark.parametrize("dist", ["exponential", "uniform", "normal"])
def test_imputed_values_follow_the_left_truncated_predictive(dist):
    """Sec. 4.2: the imputed time is a draw of p(x | x > tau).  With every worker's predictive draws
    iid from a known law the imputed values must have that law's truncated mean."""
    rng = np.random.default_rng(17)
    S, N = 2000, 4000
    if dist == "exponential":           # memoryless: E[x | x > tau] = tau + 1, sd 1
        x, tau, mean, sd = rng.exponential(1.0, (S, N)), 0.7, 1.7, 1.0
    elif dist == "uniform":             # U(tau, 1): mean (1 + tau)/2
        x, tau = rng.random((S, N)), 0.25
        mean, sd = 0.625, 0.75 / math.sqrt(12)
    else:                               # N(0,1) cut at tau: mean = pdf(tau)/sf(tau)
        x, tau = rng.standard_normal((S, N)), 1.0
        mean = stats.norm.pdf(tau) / stats.norm.sf(tau)
        sd = math.sqrt(1 + tau * mean - mean ** 2)
    u = rng.random(N).astype(np.float32)
    full, cnt = oracle.impute_censored(x.astype(np.float32), np.zeros(N, np.float32), np.ones(N, np.uint8), tau, u)
    assert np.all(cnt > 0) and np.all(full > tau)
    assert abs(full.mean() - mean) < 4 * sd / math.sqrt(N)
    assert abs(full.std() - sd) < 0.06 * sd


# ---- Elfving / the "order" baseline -----------------------------------------------

def exact_normal_order_mean(j, n, mu, sigma):
    """E[x_(j)] of n iid normals by quadrature of the integral of Sec. 3.1.1."""
    logz = math.lgamma(n + 1) - math.lgamma(j) - math.lgamma(n - j + 1)

    def f(x):
        return x * math.exp(logz + (j - 1) * stats.norm.logcdf(x) + (n - j) * stats.norm.logsf(x)) * stats.norm.pdf(x)

    val, _ = integrate.quad(f, -12, 12, epsabs=1e-12, epsrel=1e-12, limit=400)
    return mu + sigma * val


def test_elfving_reproduces_the_papers_worked_example():
    g = read_golden()
    n, mu, sd = int(g["workers"]), g["runtime_mean_s"], g["runtime_sd_s"]
    e_max = oracle.elfving_mean(n, n, mu, sd)
    # printed with rounded mu and sigma: agreement to the printed precision of those inputs
    assert abs(e_max - g["expected_max_s"]) < 5e-3
    # eq. 3: the mean idle time is about E[x_(n)] - E[x_(n/2)]
    idle = e_max - oracle.elfving_mean(n // 2, n, mu, sd)
    assert abs(idle - g["expected_idle_s"]) < 5e-3


@pytest.mark.parametrize("n", [5, 20, 158])
def test_elfving_is_close_to_the_exact_integral_and_antisymmetric(n):
    mu, sd = 1.057, 0.393
    for j in sorted({1, 2, n // 3 + 1, n // 2 + 1, n - 1, n}):
        approx = oracle.elfving_mean(j, n, mu, sd)
        exact = exact_normal_order_mean(j, n, mu, sd)
        assert abs(approx - exact) < 0.04 * sd, (j, n, approx, exact)   # Elfving's approximation error (largest at the extremes of small n)
        assert abs(approx + oracle.elfving_mean(n + 1 - j, n, mu, sd) - 2 * mu) < 1e-9
    means = [oracle.elfving_mean(j, n, mu, sd) for j in range(1, n + 1)]
    assert np.all(np.diff(means) > 0)


def test_elfving_quantile_against_the_library_inverse():
    n = 64
    pi = math.pi
    for j in range(1, n + 1):
        want = stats.norm.ppf((j - pi / 8) / (n - pi / 4 + 1))
        assert abs(oracle.elfving_mean(j, n, 0.0, 1.0) - want) < 1e-9


def test_order_cutoff_is_the_enumerated_argmax():
    for n, mu, sd in [(8, 1.0, 0.1), (158, 1.057, 0.393), (64, 2.0, 0.5)]:
        r = oracle.cutoff_elfving(n, mu, sd)
        om = np.array([c / oracle.elfving_mean(c, n, mu, sd) if oracle.elfving_mean(c, n, mu, sd) > 0 else -np.inf
                       for c in range(1, n + 1)])
        assert r["cstar"] == n - int(np.argmax(om[::-1]))
        assert np.array_equal(r["omega"], om)
    # narrow spread: waiting for everybody is best; the floor excludes non-positive predicted times
    assert oracle.cutoff_elfving(16, 1.0, 0.01)["cstar"] == 16
    r = oracle.cutoff_elfving(158, 1.057, 0.393, t_floor=0.5)
    assert np.all(r["mean"][np.isfinite(r["omega"])] > 0.5)
    assert oracle.cutoff_elfving(10, -5.0, 0.1)["status"] == oracle.NO_ELIGIBLE


# ---- throughput of a run over a trace (Fig. 2's three curves) ------------------------

def test_throughput_on_the_papers_toy_example():
    g = read_golden()
    n = 12
    row = np.concatenate([np.full(n - 2, 5.0), [g["toy_second_slowest_s"], g["toy_slowest_s"]]])
    trace = np.stack([np.random.default_rng(t).permutation(row) for t in range(7)])
    cut, sync, best = oracle.trace_throughput(trace, np.full(7, n - 1, np.int32))
    assert cut == pytest.approx((n - 1) / 8.0) and sync == pytest.approx(n / 10.0)
    # per step the wait drops from the slowest to the second slowest worker: 20 % less wall-clock
    assert 1 - 8.0 / 10.0 == pytest.approx(g["toy_wallclock_reduction"])
    brute = max(range(1, n + 1), key=lambda c: (c / np.sort(row)[c - 1], c))
    assert best == pytest.approx(brute / np.sort(row)[brute - 1])


def test_throughput_enumeration_and_bounds():
    rng = np.random.default_rng(3)
    T, N = 50, 9
    trace = rng.lognormal(0, 0.4, (T, N))
    cs = rng.integers(1, N + 1, T).astype(np.int32)
    cut, sync, best = oracle.trace_throughput(trace, cs)
    srt = np.sort(trace, axis=1)
    assert cut == pytest.approx(cs.sum() / srt[np.arange(T), cs - 1].sum())
    assert sync == pytest.approx(T * N / srt[:, -1].sum())
    g = t = 0.0
    for r in srt:
        c = max(range(1, N + 1), key=lambda c: (c / r[c - 1], c))
        g += c
        t += r[c - 1]
    assert best == pytest.approx(g / t)
    with pytest.raises(ValueError):
        oracle.trace_throughput(trace, np.zeros(T, np.int32))
