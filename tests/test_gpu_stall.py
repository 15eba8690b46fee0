"""GPU: a filter whose workgroups stop waiting for each other is reported as an error.

Wide encoders (R > 256) split the recurrence of the guide's RNNs (Sec. 3.1.3) over several
workgroups that exchange their part of the state through memory, waiting a bounded number of
polls; encoders of 129-256 units with a large input matrix wait the same way for the projection
workgroups of their launch.  The host lowers that number to zero for a few calls, so every wait counts as having run
out: every workgroup then takes the give-up path and exits normally.  The decision must come back
as DKF_ESTALLED (not as the informational CUTOFF_NO_ELIGIBLE), the separate calls must report it
through dkf_check, and the model must work again once the limit is restored.
"""
import numpy as np
import pytest

import cluster_synth as synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1803_04209_amd import api

    return api


@pytest.mark.parametrize("dtype,R,N", [("f32", 320, 96), ("bf16", 512, 96), ("f32", 256, 192)])
def test_stalled_exchange_is_an_error_and_recovers(api, dtype, R, N):
    """(R = 256 with 192 workers: one workgroup per direction, which waits for the projection
    workgroups of the same launch instead.)"""
    import torch

    cfg = synth.ClusterConfig("wide", 9, N, 4, 64 if dtype == "bf16" else 8, R if dtype == "bf16" else 40, R, 160,
                              dtype, 50, "iid_stragglers_tiny")
    blob = synth.make_blob(cfg, std=0.05)
    tr = synth.make_trace(cfg)
    eq, ez, ex = (torch.from_numpy(a).cuda() for a in synth.make_noise(cfg))
    g, ref = api.Predictor(cfg, blob), api.Predictor(cfg, blob)
    S = cfg.samples
    for t in range(cfg.lag + 1):
        c, status = g.decide(tr[t], S, eq, ez, ex)
        assert (c, status) == ref.decide(tr[t], S, eq, ez, ex)
    assert status in (api.DKF_OK, api.CUTOFF_NO_ELIGIBLE)
    assert api.dkf_check(g.handle) == api.DKF_OK

    api.dkf_set_exchange_spin_limit(g.handle, 0)
    t = cfg.lag + 1
    with pytest.raises(api.DkfError) as e:
        g.decide(tr[t], S, eq, ez, ex)
    assert e.value.code == api.DKF_ESTALLED
    assert api.dkf_check(g.handle) == api.DKF_ESTALLED
    ref.decide(tr[t], S, eq, ez, ex)
    # the separate calls: the step is enqueued, the failure shows at dkf_check, samples are NaN
    t += 1
    assert g.filter_step(tr[t]) == api.DKF_OK
    x = g.sample_runtimes(eq, ez, ex)
    assert api.dkf_check(g.handle) == api.DKF_ESTALLED
    assert bool(torch.isnan(x).all())
    ref.decide(tr[t], S, eq, ez, ex)

    # limit restored: the window took every observation, so the next decisions equal the reference's
    api.dkf_set_exchange_spin_limit(g.handle, 1 << 20)
    for t in range(cfg.lag + 3, cfg.lag + 6):
        assert g.decide(tr[t], S, eq, ez, ex) == ref.decide(tr[t], S, eq, ez, ex)
        assert api.dkf_check(g.handle) == api.DKF_OK
    assert torch.equal(g.decide_samples(S), ref.decide_samples(S))
    with pytest.raises(api.DkfError):
        api.dkf_set_exchange_spin_limit(g.handle, -1)
    g.close()
    ref.close()


def test_narrow_encoders_have_no_exchange(api):
    cfg = synth.CONFIGS["tiny"]
    g = api.Predictor(cfg, synth.make_blob(cfg))
    api.dkf_set_exchange_spin_limit(g.handle, 0)  # nothing waits on anything: no effect
    tr = synth.make_trace(cfg)
    for t in range(cfg.lag + 2):
        c, status = g.decide(tr[t], cfg.samples, seed=t)
    assert status in (api.DKF_OK, api.CUTOFF_NO_ELIGIBLE) and api.dkf_check(g.handle) == api.DKF_OK
    g.close()
