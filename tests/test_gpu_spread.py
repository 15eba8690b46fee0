"""GPU parity: cutoff_rank_spread (the +-2 sd bands of Fig. 3) against the CPU oracle.

Tolerance.  Each output is sqrt(sum / S); the sum is built from 16 fused multiply-adds per wavefront,
16 wavefront sums per 256-row segment and ceil(S / 256) segment partials, all non-negative fp32
terms, so its relative error is at most about (32 + S / 256) * 2^-24 and the root halves it: below
1e-5 for S <= 65536; 4e-5 is used
for every size.  The centre the kernel is given is the GPU's fp32 rank mean, off from the oracle's
fp64 mean by d <= a few 2^-24 |mean|; that adds d^2 to the variance, hence at most d to the sd, which
the absolute term 1e-6 * max|mean| covers (it matters only where the spread itself is ~ 0).
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


def check(api, x):
    import torch

    res = api.select_cutoff(torch.from_numpy(x).cuda(), want_sorted=True)
    sd = api.rank_spread(res["sorted"], res["mean"]).cpu().numpy()
    mean_ref, sd_ref = oracle.rank_spread(x)
    atol = 1e-6 * float(np.max(np.abs(mean_ref)))
    err = np.abs(sd - sd_ref)
    assert np.all(err <= 4e-5 * sd_ref + atol), (float(err.max()), float(sd_ref.min()), atol)
    return sd, sd_ref


@pytest.mark.parametrize("S,N", [(1, 1), (1, 70), (2, 1), (5, 3), (63, 64), (64, 65), (65, 128), (130, 256),
                                 (257, 158), (1000, 48), (4099, 130), (300, 2175), (77, 4096)])
def test_shapes_with_ragged_tails(api, S, N):
    check(api, synth.make_runtime_matrix("lognormal_stragglers", S, N, seed=S * 11 + N))


@pytest.mark.parametrize("kind", ["normal", "ties", "uniform"])
def test_value_kinds(api, kind):
    check(api, synth.make_runtime_matrix(kind, 777, 100, seed=5))


def test_no_spread_and_known_spread(api):
    row = synth.make_runtime_matrix("uniform", 1, 96, seed=1)[0]
    g = np.random.default_rng(2)
    same = np.stack([g.permutation(row) for _ in range(200)]).astype(np.float32)
    sd, _ = check(api, same)
    assert np.all(sd <= 1e-6)
    # uniform order statistics are Beta(c, N - c + 1): closed-form spread, Monte-Carlo tolerance
    S, N = 32768, 16
    x = g.random((S, N), dtype=np.float32)
    sd, _ = check(api, x)
    c = np.arange(1, N + 1)
    assert np.allclose(sd, np.sqrt(c * (N - c + 1) / ((N + 1) ** 2 * (N + 2))), rtol=0.03)


@pytest.mark.parametrize("S,N", [(4096, 128), (16384, 512), (8192, 2048)])
def test_benchmark_shapes(api, S, N):
    check(api, synth.make_runtime_matrix("lognormal_stragglers", S, N, seed=S + N))


def test_unaligned_views_take_the_narrow_path(api):
    """N divisible by 4 but a mean vector that is only 4-byte aligned."""
    import torch

    x = synth.make_runtime_matrix("normal", 500, 64, seed=8)
    res = api.select_cutoff(torch.from_numpy(x).cuda(), want_sorted=True)
    shifted = torch.empty(65, device="cuda")[1:]
    shifted.copy_(res["mean"])
    sd = api.rank_spread(res["sorted"], shifted).cpu().numpy()
    ref = api.rank_spread(res["sorted"], res["mean"]).cpu().numpy()
    assert np.allclose(sd, ref, rtol=2e-6)
    _, sd_ref = oracle.rank_spread(x)
    assert np.allclose(sd, sd_ref, rtol=4e-5)


def test_argument_errors(api):
    import torch

    x = torch.ones((8, 4), device="cuda")
    m = torch.ones(4, device="cuda")
    out = torch.empty(4, device="cuda")
    small = torch.empty(8, dtype=torch.uint8, device="cuda")
    with pytest.raises(api.DkfError) as e:
        api.cutoff_rank_spread(x, m, out, small)
    assert e.value.code == api.DKF_EINVAL
    ws = torch.empty(api.cutoff_rank_spread_workspace(8, 4), dtype=torch.uint8, device="cuda")
    api.cutoff_rank_spread(x, m, out, ws)
    torch.cuda.synchronize()
    assert torch.all(out == 0.0)
