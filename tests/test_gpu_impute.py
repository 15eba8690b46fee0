"""GPU parity: dkf_impute_censored (Sec. 4.2) against the CPU oracle, bit for bit.

The imputed value is one of the sample matrix's own entries (or tau, or the
observed time) and the count is an integer, so every output must be identical.
"""
import numpy as np
import pytest

import oracle
import cluster_synth as synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1803_04209_amd import api

    return api


def both(api, x, obs, cens, tau, u):
    import torch

    xf, cnt = api.impute_censored(torch.from_numpy(x).cuda(), torch.from_numpy(obs).cuda(),
                                  torch.from_numpy(cens).cuda(), float(tau), torch.from_numpy(u).cuda())
    of, oc = oracle.impute_censored(x, obs, cens, np.float32(tau), u)
    got = xf.cpu().numpy()
    assert np.array_equal(got.view(np.uint32), of.view(np.uint32)), "imputed vector"
    assert np.array_equal(cnt.cpu().numpy(), oc), "counts of exceeding draws"
    return got, oc


def case(S, N, seed, frac=0.3, kind="lognormal_stragglers", q=0.7):
    g = np.random.default_rng(seed)
    x = synth.make_runtime_matrix(kind, S, N, seed=seed)
    obs = synth.make_runtime_matrix(kind, 1, N, seed=seed + 1)[0]
    cens = (g.random(N) < frac).astype(np.uint8)
    tau = np.float32(np.quantile(x, q))
    u = g.random(N).astype(np.float32)
    return x, obs, cens, tau, u


@pytest.mark.parametrize("S,N", [(1, 1), (1, 70), (5, 3), (63, 64), (64, 65), (65, 128), (257, 158), (1000, 48),
                                 (4099, 130), (300, 2175)])
def test_shapes_with_ragged_tails(api, S, N):
    both(api, *case(S, N, seed=S * 7 + N))


@pytest.mark.parametrize("kind", ["normal", "ties", "signed_zeros", "uniform"])
def test_value_kinds(api, kind):
    x, obs, cens, tau, u = case(777, 100, seed=11, kind=kind)
    both(api, x, obs, cens, tau, u)
    both(api, x, obs, cens, np.float32(0.5), u)   # for "ties": many draws equal tau exactly, none of them exceeds it
    both(api, x, obs, cens, np.float32(-0.0), u)


def test_all_none_and_extreme_u(api):
    x, obs, cens, tau, u = case(500, 90, seed=3)
    both(api, x, obs, np.ones_like(cens), tau, u)
    got, _ = both(api, x, obs, np.zeros_like(cens), tau, u)
    assert np.array_equal(got, obs)
    both(api, x, obs, np.ones_like(cens), tau, np.zeros_like(u))
    both(api, x, obs, np.ones_like(cens), tau, np.full_like(u, np.nextafter(np.float32(1), np.float32(0))))
    # nothing exceeds tau: every dropped worker gets tau
    got, cnt = both(api, x, obs, np.ones_like(cens), np.float32(x.max()), u)
    assert np.all(got == x.max()) and np.all(cnt == 0)
    # infinities in the matrix are ordinary values
    x[::7, ::5] = np.inf
    x[3::11, 1::4] = -np.inf
    both(api, x, obs, np.ones_like(cens), tau, u)


@pytest.mark.parametrize("S,N", [(4096, 128), (16384, 512), (8192, 2048)])
def test_benchmark_shapes(api, S, N):
    both(api, *case(S, N, seed=S + N, frac=0.5, q=0.9))


def test_argument_errors(api):
    import torch

    S, N = 8, 4
    x = torch.ones((S, N), device="cuda")
    v = torch.ones(N, device="cuda")
    c = torch.ones(N, dtype=torch.uint8, device="cuda")
    out = torch.empty(N, device="cuda")
    small = torch.empty(4, dtype=torch.uint8, device="cuda")
    with pytest.raises(api.DkfError) as e:
        api.dkf_impute_censored(x, v, c, 0.5, v, out, None, small)
    assert e.value.code == api.DKF_EINVAL
    ws = torch.empty(api.dkf_impute_workspace(S, N), dtype=torch.uint8, device="cuda")
    with pytest.raises(api.DkfError):
        api.dkf_impute_censored(x, v, c, float("nan"), v, out, None, ws)
    assert api.dkf_impute_workspace(0, 4) == 0
    api.dkf_impute_censored(x, v, c, 0.5, v, out, None, ws)   # n_exceed is optional
    torch.cuda.synchronize()
    assert torch.all(out == 1.0)


def test_online_loop_with_censored_feedback(api):
    """Alg. 1 with Sec. 4.2: decide, wait for the c* fastest workers of the real iteration, impute the
    rest from the decision's own samples, feed the completed vector to the filter.  The GPU loop and
    the oracle's loop are given the same samples (the GPU's) at every step."""
    import torch

    cfg = synth.CONFIGS["tiny"]
    blob = synth.make_blob(cfg)
    trace = synth.make_trace(cfg)
    gpu = api.Predictor(cfg, blob)
    rng = np.random.default_rng(9)
    N, L, S = cfg.n_workers, cfg.lag, cfg.samples
    dropped_total = 0
    x_in = trace[0]
    for t in range(L + 25):
        c, status = gpu.decide(x_in, S, seed=1000 + t)
        if status == api.DKF_WARMUP:      # no prediction yet: fully synchronous step, nothing censored
            assert c == N
            x_in = trace[t + 1]
            continue
        nxt = trace[t + 1]
        order = np.argsort(nxt, kind="stable")
        tau = np.float32(nxt[order[c - 1]])
        cens = np.ones(N, np.uint8)
        cens[order[:c]] = 0
        u = rng.random(N).astype(np.float32)
        samples = gpu.decide_samples(S)
        xf, cnt = api.impute_censored(samples, torch.from_numpy(nxt).cuda(), torch.from_numpy(cens).cuda(),
                                      float(tau), torch.from_numpy(u).cuda())
        of, oc = oracle.impute_censored(samples.cpu().numpy(), nxt, cens, tau, u)
        assert np.array_equal(xf.cpu().numpy().view(np.uint32), of.view(np.uint32))
        assert np.array_equal(cnt.cpu().numpy(), oc)
        filled = xf.cpu().numpy()
        assert np.all(filled[cens == 1] >= tau) and np.array_equal(filled[cens == 0], nxt[cens == 0])
        dropped_total += int(cens.sum())
        x_in = filled   # positive and finite, since tau > 0
    gpu.close()
    assert dropped_total > 0
