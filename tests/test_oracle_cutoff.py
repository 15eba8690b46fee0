"""Pins for the oracle's order-statistics / cutoff stage (CPU only).

Each test checks the oracle against something fixed by the paper or by
mathematics, not against itself: closed-form order statistics, quadrature of
the integral in Sec. 3.1.1, brute force over every cutoff, and the worked
examples the paper prints (tests/golden/paper_worked_examples.txt).
"""
import itertools
import math

import numpy as np
import pytest
from scipy import integrate, stats

import oracle
import cluster_synth as synth


def read_golden(path):
    out = {}
    for line in path.read_text().splitlines():
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = float(v)
    return out


# ---- sort -------------------------------------------------------------------

@pytest.mark.parametrize("kind", ["normal", "lognormal_stragglers", "ties", "signed_zeros"])
@pytest.mark.parametrize("N", [1, 2, 7, 16, 100])
def test_sorted_rows_and_permutation(kind, N):
    x = synth.make_runtime_matrix(kind, 37, N, seed=11 + N)
    r = oracle.cutoff_select(x, t_floor=-np.inf)
    srt, perm = r["sorted"], r["perm"]
    assert np.all(np.diff(srt, axis=1) >= 0)
    assert np.array_equal(np.sort(perm, axis=1), np.tile(np.arange(N), (37, 1)))
    gathered = np.take_along_axis(x, perm, axis=1)
    assert np.array_equal(gathered.view(np.uint32), srt.astype(np.float32).view(np.uint32))
    # values agree with the library sort (sign of zero aside, which np.sort does not order)
    assert np.array_equal(np.sort(x.astype(np.float64), axis=1), srt)


def test_tie_order_is_negative_zero_then_index():
    x = np.array([[0.0, 1.0, -0.0, 1.0, -0.0, 0.0, -1.0]], dtype=np.float32)
    r = oracle.cutoff_select(x, t_floor=-np.inf)
    assert r["perm"][0].tolist() == [6, 2, 4, 0, 5, 1, 3]
    assert np.signbit(r["sorted"][0]).tolist() == [True, True, True, False, False, False, False]


def test_every_permutation_of_six():
    base = np.array([0.5, 1.5, 2.5, 3.5, 4.5, 5.5])
    rows = np.array(list(itertools.permutations(base)), dtype=np.float32)
    r = oracle.cutoff_select(rows)
    assert np.array_equal(r["sorted"], np.tile(base, (720, 1)))
    inv = np.argsort(rows, axis=1, kind="stable")
    assert np.array_equal(r["perm"], inv)


# ---- per-rank means against closed forms --------------------------------------

def test_uniform_order_statistics():
    # E[x_(c)] = c/(N+1), Var = c(N+1-c)/((N+1)^2 (N+2)) for iid U(0,1)
    S, N = 20000, 24
    x = synth.make_runtime_matrix("uniform", S, N, seed=5)
    mean = oracle.cutoff_select(x)["mean"]
    c = np.arange(1, N + 1)
    sd = np.sqrt(c * (N + 1 - c) / ((N + 1) ** 2 * (N + 2) * S))
    assert np.all(np.abs(mean - c / (N + 1)) < 4.5 * sd)


def test_exponential_order_statistics_and_cutoff():
    # E[x_(c)] = sum_{i=N-c+1}^{N} 1/i (Renyi); Omega(c) then strictly decreases, so c* = 1
    S, N = 20000, 20
    x = synth.make_runtime_matrix("exponential", S, N, seed=6)
    r = oracle.cutoff_select(x)
    c = np.arange(1, N + 1)
    expect = np.array([sum(1.0 / i for i in range(N - k + 1, N + 1)) for k in c])
    sd = np.sqrt(np.array([sum(1.0 / i ** 2 for i in range(N - k + 1, N + 1)) for k in c]) / S)
    assert np.all(np.abs(r["mean"] - expect) < 4.5 * sd)
    assert r["cstar"] == 1
    assert np.all(np.diff(r["omega"]) < 0)


def normal_order_stat_mean(n, j, mu, sigma):
    """Quadrature of Z(n,j) int x Phi^{j-1} (1-Phi)^{n-j} p dx (Sec. 3.1.1)."""
    logz = math.lgamma(n + 1) - math.lgamma(j) - math.lgamma(n - j + 1)

    def f(u):
        lp = (j - 1) * stats.norm.logcdf(u) + (n - j) * stats.norm.logsf(u) + stats.norm.logpdf(u)
        return u * math.exp(logz + lp)

    val, _ = integrate.quad(f, -12, 12, limit=400)
    return mu + sigma * val


def test_normal_order_statistics_match_the_integral():
    S, N = 20000, 12
    mu, sigma = 1.5, 0.25
    x = (mu + sigma * synth.make_runtime_matrix("normal", S, N, seed=7)).astype(np.float32)
    r = oracle.cutoff_select(x)
    expect = np.array([normal_order_stat_mean(N, j, mu, sigma) for j in range(1, N + 1)])
    assert np.all(np.abs(r["mean"] - expect) < 5 * sigma / math.sqrt(S))
    assert np.all(np.diff(r["mean"]) >= 0)  # E[x_(1)] <= ... <= E[x_(n)]


def test_paper_worked_example_158_workers(golden_dir):
    g = read_golden(golden_dir / "paper_worked_examples.txt")
    n, mu, sd = int(g["workers"]), g["runtime_mean_s"], g["runtime_sd_s"]
    S = 40000
    x = (mu + sd * synth.make_runtime_matrix("normal", S, n, seed=158)).astype(np.float32)
    mean = oracle.cutoff_select(x, t_floor=-np.inf)["mean"]
    # the paper's figures come from the Elfving approximation (a few 1e-3 off the exact value)
    assert abs(mean[-1] - g["expected_max_s"]) < 1.5e-2
    idle = np.mean(mean[-1] - mean)
    assert abs(idle - g["expected_idle_s"]) < 1.5e-2
    # eq. 3: the idle time is close to E[x_(n)] - E[x_(n/2)]
    assert abs(idle - (mean[-1] - mean[n // 2 - 1])) < 1e-2
    # exact value of the maximum by quadrature
    assert abs(mean[-1] - normal_order_stat_mean(n, n, mu, sd)) < 5 * sd * 0.45 / math.sqrt(S) + 1e-3


# ---- Omega and the argmax ---------------------------------------------------

def brute_force(x, c_min, c_max, t_floor):
    srt = np.sort(x.astype(np.float64), axis=1)
    best, best_c = None, None
    for c in range(c_min, c_max + 1):
        m = math.fsum(srt[:, c - 1]) / x.shape[0]
        if m > t_floor:
            om = c / m
            if best is None or om >= best:
                best, best_c = om, c
    return best_c, best


@pytest.mark.parametrize("N", [1, 2, 3, 5, 8])
@pytest.mark.parametrize("seed", range(6))
def test_argmax_by_enumeration(N, seed):
    kind = ["lognormal_stragglers", "normal", "exponential"][seed % 3]
    x = synth.make_runtime_matrix(kind, 9, N, seed=1000 + seed)
    r = oracle.cutoff_select(x)
    c, om = brute_force(x, 1, N, 0.0)
    if c is None:
        assert r["status"] == oracle.NO_ELIGIBLE and r["cstar"] == N
    else:
        assert r["status"] == oracle.OK
        assert 1 <= r["cstar"] <= N
        assert r["omega"][r["cstar"] - 1] == pytest.approx(om, rel=1e-12)
        assert r["cstar"] == c


def test_paper_toy_straggler(golden_dir):
    g = read_golden(golden_dir / "paper_worked_examples.txt")
    n = 10
    row = np.full(n, 7.0)
    row[3], row[8] = g["toy_slowest_s"], g["toy_second_slowest_s"]
    r = oracle.cutoff_select(row[None, :].astype(np.float32))
    # waiting for n-1 instead of n shortens the step by the printed fraction
    assert 1 - r["mean"][n - 2] / r["mean"][n - 1] == pytest.approx(g["toy_wallclock_reduction"])
    assert r["omega"][n - 2] / r["omega"][n - 1] == pytest.approx((n - 1) * 10.0 / (8.0 * n))
    assert r["cstar"] == n - 2  # eight workers at 7 s beat both stragglers: 8/7 > 9/8 > 10/10
    assert r["perm"][0, -1] == 3 and r["perm"][0, -2] == 8


def test_exact_ties_go_to_the_largest_cutoff():
    N = 12
    row = 0.25 * np.arange(1, N + 1)  # Omega(c) = 4 for every c, exactly
    r = oracle.cutoff_select(np.tile(row, (3, 1)).astype(np.float32))
    assert np.all(r["omega"] == 4.0)
    assert r["cstar"] == N


def test_floor_bounds_and_no_eligible():
    x = synth.make_runtime_matrix("normal", 64, 10, seed=3)  # about half the ranks have negative means
    r = oracle.cutoff_select(x)
    neg = r["mean"] <= 0
    assert neg.any() and (~neg).any()
    assert np.all(np.isneginf(r["omega"][neg])) and np.all(np.isfinite(r["omega"][~neg]))
    assert not neg[r["cstar"] - 1]
    r2 = oracle.cutoff_select(x - 100.0)
    assert r2["status"] == oracle.NO_ELIGIBLE and r2["cstar"] == 10
    r3 = oracle.cutoff_select(x - 100.0, c_min=2, c_max=7)
    assert r3["status"] == oracle.NO_ELIGIBLE and r3["cstar"] == 7
    y = synth.make_runtime_matrix("lognormal_stragglers", 64, 10, seed=4)
    r4 = oracle.cutoff_select(y, c_min=3, c_max=6)
    assert 3 <= r4["cstar"] <= 6
    assert np.all(np.isneginf(r4["omega"][:2])) and np.all(np.isneginf(r4["omega"][6:]))
    assert r4["cstar"] == brute_force(y, 3, 6, 0.0)[0]
    for bad in [dict(c_min=0), dict(c_max=11), dict(c_min=5, c_max=4)]:
        with pytest.raises(ValueError):
            oracle.cutoff_select(y, **bad)


def test_scale_and_relabelling_invariance():
    x = synth.make_runtime_matrix("lognormal_stragglers", 200, 33, seed=9)
    r = oracle.cutoff_select(x)
    assert oracle.cutoff_select(x * np.float32(4.0))["cstar"] == r["cstar"]  # exact power-of-two scaling
    p = np.random.default_rng(0).permutation(33)
    rp = oracle.cutoff_select(np.ascontiguousarray(x[:, p]))
    assert rp["cstar"] == r["cstar"]
    assert np.array_equal(rp["sorted"], r["sorted"])
    assert np.array_equal(p[rp["perm"]], r["perm"]) or np.array_equal(
        np.take_along_axis(x, r["perm"], 1), np.take_along_axis(x[:, p], rp["perm"], 1))


def test_f64_and_f32_entries_agree():
    x = synth.make_runtime_matrix("lognormal_stragglers", 50, 17, seed=10)
    a = oracle.cutoff_select(x)
    b = oracle.cutoff_select(x.astype(np.float64))
    assert a["cstar"] == b["cstar"] and np.array_equal(a["perm"], b["perm"]) and np.array_equal(a["mean"], b["mean"])


# ---- the other reading of Omega: the mean of c / x_(c) (Sec. 3) -----------------------------------

def test_rate_rule_hand_worked_and_degenerate_cases():
    # two rows (1, 2) and (4, 2): rank 1 -> (1/1 + 1/2)/2 = 3/4, rank 2 -> (1/2 + 1/4)/2 = 3/8;
    # Omega = (3/4, 2 * 3/8): an exact tie, which goes to the larger cutoff
    r = oracle.cutoff_select_rate(np.array([[1.0, 2.0], [4.0, 2.0]]))
    assert np.array_equal(r["rate"], [0.75, 0.375]) and np.array_equal(r["omega"], [0.75, 0.75])
    assert (r["cstar"], r["status"]) == (2, oracle.OK)
    # identical rows: the mean of the ratio is the ratio of the mean
    x = np.tile(np.array([[3.0, 1.0, 2.0, 8.0]]), (5, 1))
    a, b = oracle.cutoff_select_rate(x), oracle.cutoff_select(x)
    assert np.allclose(a["omega"], b["omega"], rtol=1e-15) and a["cstar"] == b["cstar"]
    # a rank with one non-positive sample is out, for good: rank 1 here
    x = np.array([[0.5, 1.0, 2.0], [-0.1, 1.0, 3.0]])
    r = oracle.cutoff_select_rate(x)
    assert np.isinf(r["rate"][0]) and np.isneginf(r["omega"][0]) and r["cstar"] in (2, 3)
    r = oracle.cutoff_select_rate(-x)
    assert (r["cstar"], r["status"]) == (3, oracle.NO_ELIGIBLE)
    with pytest.raises(ValueError):
        oracle.cutoff_select_rate(x, t_floor=-1.0)


def test_rate_rule_uniform_order_statistics():
    # x_(c) of N iid U(0,1) is Beta(c, N + 1 - c), whose reciprocal has mean N / (c - 1) and second
    # moment N (N - 1) / ((c - 1)(c - 2)): Omega(c) = c N / (c - 1) for c >= 3 within 5 standard errors
    S, N = 40000, 12
    x = np.random.default_rng(3).random((S, N))
    r = oracle.cutoff_select_rate(x, c_min=3)
    c = np.arange(3, N + 1)
    mean = N / (c - 1)
    var = N * (N - 1) / ((c - 1) * (c - 2)) - mean ** 2
    assert np.all(np.abs(r["rate"][2:] - mean) < 5 * np.sqrt(var / S))
    assert r["cstar"] == 3  # c N / (c - 1) falls with c


def test_rate_rule_against_enumeration_and_jensen():
    rng = np.random.default_rng(8)
    for S, N in [(1, 1), (7, 5), (50, 8)]:
        x = rng.lognormal(0.0, 0.5, (S, N))
        for c_min, c_max in [(1, N), (min(2, N), N), (1, max(1, N - 1))]:
            r = oracle.cutoff_select_rate(x, c_min=c_min, c_max=c_max)
            srt = np.sort(x, axis=1)
            om = np.array([np.mean(c / srt[:, c - 1]) if c_min <= c <= c_max else -np.inf for c in range(1, N + 1)])
            assert np.allclose(r["omega"], om, rtol=1e-13)
            assert r["cstar"] == max(c for c in range(1, N + 1) if om[c - 1] == om.max())
        # the mean of the ratio is never below the ratio of the mean (Jensen, 1/x convex on x > 0)
        assert np.all(oracle.cutoff_select_rate(x)["omega"] >= oracle.cutoff_select(x)["omega"] * (1 - 1e-12))
