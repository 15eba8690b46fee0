"""GPU parity at the edges of what dkf_load_weights accepts.

The header's limits are N <= 4096, L <= 256, Z, H, R <= 1024 and the staged guide kernel's LDS bound
(fp32: 648 Zp + 132 max(Rp, Hp) <= 147456 with sizes rounded up to 32; bf16: 516 Zp + 66 max(Rp, Hp)
<= 147456 with sizes rounded up to 64).  Each case sits on one of those edges; every stage is
compared with the oracle as in test_gpu_model.py.  Weight scales keep the ReLU recurrences
contracting (spectral radius about std * sqrt(R / 2) < 1).
"""
from dataclasses import replace

import numpy as np
import pytest

import cluster_synth as synth
from test_gpu_model import TOL, TOL_BF16, api, compare_stages, custom, make_pair  # noqa: F401

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg,std", [
    (custom(N=96, L=3, Z=64, H=800, R=800, S=40), 0.03),     # widest hidden layers fp32 takes with Z = 64
    (custom(N=200, L=4, Z=160, H=160, R=160, S=40), 0.06),   # widest latent fp32 takes with H = R = Z
    (custom(N=4096, L=2, Z=16, H=64, R=64, S=33), 0.05),     # widest row
    (replace(custom(N=16, L=256, Z=8, H=16, R=24, S=40), trace_len=300), 0.1),       # longest window, encoder in registers
    (replace(custom(N=16, L=256, Z=8, H=16, R=72, S=40), trace_len=300), 0.1),       # longest window, matrix streamed every step
], ids=["H800", "Z160", "N4096", "L256", "L256-stream"])
def test_fp32_limits(api, cfg, std):
    g, o, _ = make_pair(api, cfg, std=std)
    compare_stages(api, cfg, g, o, tol=TOL)
    g.close()


@pytest.mark.parametrize("cfg,std", [
    (custom(N=128, L=2, Z=64, H=1024, R=1024, S=40), 0.03),  # the documented maximum widths
    (custom(N=100, L=3, Z=192, H=192, R=192, S=40), 0.06),   # widest latent bf16 takes with H = R = Z
    (custom(N=4096, L=2, Z=16, H=64, R=64, S=33), 0.05),
], ids=["H1024", "Z192", "N4096"])
def test_bf16_limits(api, cfg, std):
    g, o, _ = make_pair(api, cfg, std=std, mlp_dtype=api.DKF_DTYPE_BF16)
    _, errs = compare_stages(api, cfg, g, o, tol=TOL_BF16)
    assert errs["ctx"] <= TOL
    g.close()


@pytest.mark.parametrize("kw", [dict(Z=64, H=832, R=64), dict(Z=192, H=192, R=192), dict(Z=1025), dict(H=1025),
                                dict(R=1025), dict(N=4097), dict(L=257)],
                         ids=["H832", "Z192", "Z1025", "H1025", "R1025", "N4097", "L257"])
def test_sizes_beyond_the_limits_are_refused(api, kw):
    cfg = custom(**{**dict(N=8, L=2, Z=8, H=8, R=8, S=8), **kw})
    with pytest.raises(api.DkfError) as e:
        api.Predictor(cfg, synth.make_blob(cfg))
    assert e.value.code == api.DKF_EUNSUPPORTED


def test_one_sample_and_exactly_max_samples(api):
    import torch

    cfg = custom(N=70, L=3, Z=12, H=40, R=36, S=1)
    g, o, _ = make_pair(api, cfg, std=0.3)
    x, _ = compare_stages(api, cfg, g, o)
    res = api.select_cutoff(x)
    assert res["status"] == api.DKF_OK and 1 <= res["cstar"] <= cfg.n_workers
    g.close()
    cfg = synth.CONFIGS["tiny"]
    g, o, _ = make_pair(api, cfg)
    compare_stages(api, cfg, g, o, S=cfg.samples)          # S == max_samples
    out = torch.empty((cfg.samples + 1, cfg.n_workers), device="cuda")
    eq, ez, ex = [torch.from_numpy(a).cuda() for a in synth.make_noise(cfg, cfg.samples + 1)]
    with pytest.raises(api.DkfError) as e:
        api.dkf_sample_runtimes(g.handle, cfg.samples + 1, eq, ez, ex, 0, out)
    assert e.value.code == api.DKF_EINVAL
    g.close()
