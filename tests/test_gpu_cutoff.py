"""GPU parity: cutoff_select (row sort, rank means, Omega, argmax) against the CPU oracle.

Sorted values and permutations must be bit-exact.  Rank means: the kernel adds
at most a few rows per lane in fp32 before switching to fp64, so they must
agree within 2e-6 of the rank's mean magnitude.  c* must equal the oracle's or
lie in the 1e-6 relative tie band of the oracle's Omega.
"""
import numpy as np
import pytest

import oracle
import cluster_synth as synth
from gpu_util import cstar_in_tie_band

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1803_04209_amd import api

    return api


def run_both(api, x, **kw):
    import torch

    xd = torch.from_numpy(x).cuda()
    g = api.select_cutoff(xd, want_sorted=True, want_perm=True, **kw)
    o = oracle.cutoff_select(x, **kw)
    return g, o


def check(api, x, **kw):
    g, o = run_both(api, x, **kw)
    srt = g["sorted"].cpu().numpy()
    perm = g["perm"].cpu().numpy()
    assert np.array_equal(srt.view(np.uint32), o["sorted"].astype(np.float32).view(np.uint32)), "sorted values"
    assert np.array_equal(perm, o["perm"]), "permutation"
    mean = g["mean"].cpu().numpy().astype(np.float64)
    mag = np.abs(o["sorted"]).mean(axis=0)
    tol = 2e-6 * np.maximum(mag, 1e-30)
    fin_m = np.isfinite(o["mean"])
    assert np.array_equal(mean[~fin_m], o["mean"][~fin_m]), "infinite rank means"
    assert np.all(np.abs(mean[fin_m] - o["mean"][fin_m]) <= tol[fin_m] + 1e-7 * np.abs(o["mean"][fin_m])), "rank means"
    assert g["status"] == o["status"]
    assert cstar_in_tie_band(g["cstar"], o), (g["cstar"], o["cstar"])
    om = g["omega"].cpu().numpy().astype(np.float64)
    t_floor = kw.get("t_floor", 0.0)
    with np.errstate(invalid="ignore"):
        clear = ~(np.abs(o["mean"] - t_floor) <= 10 * tol)  # away from the eligibility edge
    assert np.array_equal(np.isneginf(om[clear]), np.isneginf(o["omega"][clear]))
    fin = clear & np.isfinite(o["omega"])
    assert np.allclose(om[fin], o["omega"][fin], rtol=5e-6)
    # same call without the optional outputs gives the same decision
    import torch

    g2 = api.select_cutoff(torch.from_numpy(x).cuda(), **kw)
    # (the call without them may run a workgroup shape of its own, which adds the rows in another order)
    assert cstar_in_tie_band(g2["cstar"], o), (g2["cstar"], o["cstar"])
    assert torch.allclose(g2["mean"], g["mean"], rtol=1e-6, atol=0.0, equal_nan=True)
    return g, o


@pytest.mark.parametrize("N", [1, 2, 3, 8, 9, 16, 31, 64, 100, 128, 158, 257, 512, 1000, 1024, 2048, 2175, 4096])
def test_widths(api, N):
    S = 67 if N > 1024 else 301
    x = synth.make_runtime_matrix("lognormal_stragglers", S, N, seed=N)
    check(api, x)


@pytest.mark.parametrize("kind", ["normal", "ties", "signed_zeros", "uniform", "exponential"])
@pytest.mark.parametrize("S,N", [(1, 16), (5, 128), (1000, 48), (4099, 128), (130, 512)])
def test_kinds_and_ragged_sample_counts(api, kind, S, N):
    x = synth.make_runtime_matrix(kind, S, N, seed=S + N)
    check(api, x, t_floor=-np.inf if kind in ("normal", "signed_zeros") else 0.0)
    if kind == "normal":
        check(api, x)  # about half the ranks fall under the floor


def test_infinities_and_bounds(api):
    x = synth.make_runtime_matrix("lognormal_stragglers", 64, 40, seed=2)
    x[3, 5] = np.inf
    x[7, 0] = -np.inf
    g, o = check(api, x, t_floor=-np.inf)
    check(api, x, c_min=7, c_max=7)
    check(api, x, c_min=3, c_max=30, t_floor=0.9)
    g, o = check(api, x - 100.0)  # the +inf keeps the last rank eligible: Omega = 40 / inf = 0
    assert g["status"] == 0 and g["cstar"] == 40
    y = synth.make_runtime_matrix("lognormal_stragglers", 64, 40, seed=2) - 100.0
    g, o = check(api, y)
    assert g["status"] == 2 and g["cstar"] == 40
    g, o = check(api, y, c_min=2, c_max=9)
    assert g["status"] == 2 and g["cstar"] == 9


def test_exact_ties_in_omega_take_the_largest(api):
    N = 96
    x = np.tile(0.25 * np.arange(1, N + 1, dtype=np.float32), (8, 1))
    rng = np.random.default_rng(0)
    x = np.stack([r[rng.permutation(N)] for r in x])
    g, o = check(api, x)
    assert g["cstar"] == N == o["cstar"]


def test_closed_forms_on_the_gpu(api):
    import torch

    S, N = 20000, 24
    x = synth.make_runtime_matrix("uniform", S, N, seed=5)
    g = api.select_cutoff(torch.from_numpy(x).cuda())
    c = np.arange(1, N + 1)
    sd = np.sqrt(c * (N + 1 - c) / ((N + 1) ** 2 * (N + 2) * S))
    assert np.all(np.abs(g["mean"].cpu().numpy() - c / (N + 1)) < 4.5 * sd + 1e-6)
    x = synth.make_runtime_matrix("exponential", S, N, seed=6)
    assert api.select_cutoff(torch.from_numpy(x).cuda())["cstar"] == 1


def test_argument_errors(api):
    import torch

    x = torch.ones((4, 8), device="cuda")
    for kw in (dict(c_min=0), dict(c_max=9), dict(c_min=5, c_max=4), dict(t_floor=float("nan"))):
        with pytest.raises(api.DkfError) as e:
            api.select_cutoff(x, **kw)
        assert e.value.code == api.DKF_EINVAL
    with pytest.raises(api.DkfError):
        api.select_cutoff(torch.ones((4, 5000), device="cuda"))
    ws = torch.empty(16, dtype=torch.uint8, device="cuda")
    out = torch.zeros(2, dtype=torch.int32, device="cuda")
    with pytest.raises(api.DkfError):
        api.cutoff_select(x, 1, 8, 0.0, None, None, None, None, out, ws)


def test_deterministic(api):
    import torch

    x = torch.from_numpy(synth.make_runtime_matrix("lognormal_stragglers", 16384, 512, seed=1)).cuda()
    a = api.select_cutoff(x, want_sorted=True)
    b = api.select_cutoff(x, want_sorted=True)
    assert torch.equal(a["mean"], b["mean"]) and torch.equal(a["sorted"], b["sorted"]) and a["cstar"] == b["cstar"]


@pytest.mark.parametrize("S,N", [(4096, 128), (16384, 512), (8192, 2048), (4096, 512)])
def test_benchmark_shapes(api, S, N):
    """Full preset sizes: permutation and values on sampled rows, means and c* on everything."""
    import torch

    x = synth.make_runtime_matrix("lognormal_stragglers", S, N, seed=S ^ N)
    xd = torch.from_numpy(x).cuda()
    g = api.select_cutoff(xd, want_sorted=True, want_perm=True)
    rows = np.random.default_rng(S).choice(S, 256, replace=False)
    o_rows = oracle.cutoff_select(np.ascontiguousarray(x[rows]))
    assert np.array_equal(g["sorted"][rows].cpu().numpy().view(np.uint32),
                          o_rows["sorted"].astype(np.float32).view(np.uint32))
    assert np.array_equal(g["perm"][rows].cpu().numpy(), o_rows["perm"])
    srt = g["sorted"].cpu().numpy()
    assert np.all(np.diff(srt, axis=1) >= 0)
    o = oracle.cutoff_select(x, want_sorted=False, want_perm=False)
    mean = g["mean"].cpu().numpy().astype(np.float64)
    assert np.all(np.abs(mean - o["mean"]) <= 2e-6 * np.abs(o["mean"]) + 1e-12)
    assert cstar_in_tie_band(g["cstar"], o)
    g2 = api.select_cutoff(xd)  # the read-only configuration the benchmark times
    mean2 = g2["mean"].cpu().numpy().astype(np.float64)
    assert np.all(np.abs(mean2 - o["mean"]) <= 2e-6 * np.abs(o["mean"]) + 1e-12) and cstar_in_tie_band(g2["cstar"], o)
    # (the read-only call runs a workgroup shape of its own, which adds the rows in another order)
    assert torch.allclose(g2["mean"], g["mean"], rtol=1e-6, atol=0.0)
    g3 = api.select_cutoff(xd)
    assert g3["cstar"] == g2["cstar"] and torch.equal(g3["mean"], g2["mean"])  # the same call twice: bit-identical


@pytest.mark.parametrize("kind", ["lognormal_stragglers", "normal", "uniform"])
@pytest.mark.parametrize("S,N", [(1, 16), (1000, 48), (4099, 128), (130, 512), (67, 2048), (33, 158)])
def test_rate_rule(api, kind, S, N):
    """cutoff_select_rate: Omega(c) = mean over the rows of c / x_(c).  Reciprocals are taken in fp32
    (correctly rounded) and summed like the rank sums, so the rates agree with the fp64 oracle to
    3e-6; a rank with a value at or below the floor is out on both sides; sorting is unchanged."""
    import torch

    x = synth.make_runtime_matrix(kind, S, N, seed=3 * S + N)
    if kind == "uniform":
        x = x + np.float32(0.25)  # keep the reciprocals of the lowest ranks well conditioned
    for kw in (dict(), dict(c_min=min(2, N), c_max=max(min(2, N), N - 1), t_floor=0.5)):
        g = api.select_cutoff(torch.from_numpy(x).cuda(), want_sorted=True, want_perm=True, rate=True, **kw)
        o = oracle.cutoff_select_rate(x, **kw)
        ref = oracle.cutoff_select(x, t_floor=-np.inf)
        assert np.array_equal(g["sorted"].cpu().numpy().view(np.uint32), ref["sorted"].astype(np.float32).view(np.uint32))
        assert np.array_equal(g["perm"].cpu().numpy(), ref["perm"])
        rate = g["mean"].cpu().numpy().astype(np.float64)
        fin = np.isfinite(o["rate"])
        assert np.array_equal(np.isposinf(rate), ~fin)
        assert np.allclose(rate[fin], o["rate"][fin], rtol=3e-6, atol=0)
        om = g["omega"].cpu().numpy().astype(np.float64)
        assert np.array_equal(np.isneginf(om), np.isneginf(o["omega"]))
        ok = np.isfinite(o["omega"])
        assert np.allclose(om[ok], o["omega"][ok], rtol=3e-6, atol=0)
        assert g["status"] == o["status"]
        assert cstar_in_tie_band(g["cstar"], o, rel=6e-6) if o["status"] == oracle.OK else g["cstar"] == o["cstar"]


def test_rate_rule_argument_errors(api):
    import torch

    x = torch.ones((4, 8), device="cuda")
    with pytest.raises(api.DkfError) as e:
        api.select_cutoff(x, rate=True, t_floor=-0.5)
    assert e.value.code == api.DKF_EINVAL
    with pytest.raises(api.DkfError):
        api.select_cutoff(x, rate=True, t_floor=float("nan"))


@pytest.mark.parametrize("S,N", [(300, 16), (257, 158), (4096, 512), (512, 2048)])
def test_workspace_contents_do_not_matter(api, S, N):
    """The caller's workspace may hold anything: the counter of finished workgroups and the
    candidates in it are written before they are read in every call.  Same decision from a
    workspace of all-ones bits, of zeros, and from one the previous call left behind."""
    import torch

    x = synth.make_runtime_matrix("lognormal_stragglers", S, N, seed=7 * S + N)
    o = oracle.cutoff_select(x, want_sorted=False, want_perm=False)
    xd = torch.from_numpy(x).cuda()
    ws = torch.empty(api.cutoff_select_workspace(S, N), dtype=torch.uint8, device="cuda")
    mean = torch.empty(N, dtype=torch.float32, device="cuda")
    omega = torch.empty(N, dtype=torch.float32, device="cuda")
    results = []
    for fill in (0xFF, 0x00, None, None):
        if fill is not None:
            ws.fill_(fill)
        cstar = torch.full((2,), -7, dtype=torch.int32, device="cuda")
        api.cutoff_select(xd, 1, N, 0.0, None, None, mean, omega, cstar, ws)
        c = cstar.cpu()
        results.append((int(c[0]), int(c[1]), mean.clone()))
        assert cstar_in_tie_band(int(c[0]), o)
    for r in results[1:]:
        assert r[0] == results[0][0] and r[1] == results[0][1] and torch.equal(r[2], results[0][2])


@pytest.mark.parametrize("N", [8, 16, 32, 64, 128, 256, 512, 1024, 2048, 4096])
@pytest.mark.parametrize("S", [1024, 8192])
def test_read_only_call_at_every_network_width(api, S, N):
    """Rows that fill the sorting network exactly, in numbers that divide evenly over the grid: the
    read-only call (no sorted rows, no permutation: what a decision runs) takes the loop body
    without row or column checks at every width, two rows per wavefront at 512 keys and 8192 rows.
    Means against the fp64 oracle, c* in its tie band, and the rows themselves through the
    general body."""
    import torch

    x = synth.make_runtime_matrix("lognormal_stragglers", S, N, seed=31 * S + N)
    x[3 % S, : min(N, 5)] = [0.0, -0.0, np.inf, -np.inf, 1e-30][: min(N, 5)]
    o = oracle.cutoff_select(x, want_sorted=False, want_perm=False)
    xd = torch.from_numpy(x).cuda()
    g = api.select_cutoff(xd)
    mean = g["mean"].cpu().numpy().astype(np.float64)
    fin = np.isfinite(o["mean"])
    assert np.array_equal(mean[~fin], o["mean"][~fin])
    assert np.all(np.abs(mean[fin] - o["mean"][fin]) <= 2e-6 * np.abs(o["mean"][fin]) + 1e-12)
    assert cstar_in_tie_band(g["cstar"], o)
    full = api.select_cutoff(xd, want_sorted=True)
    assert torch.allclose(g["mean"], full["mean"], rtol=1e-6, atol=0.0, equal_nan=True)
    rows = np.random.default_rng(N).choice(S, 64, replace=False)
    assert np.array_equal(full["sorted"][rows].cpu().numpy().view(np.uint32),
                          np.sort(x[rows], axis=1).view(np.uint32))
