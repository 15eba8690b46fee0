"""GPU: cutoff_select_static (the entry point that allocates nothing) against cutoff_select.

The two share their kernels; the static variant keeps the per-block rank sums in a fixed device
array of the library instead of a caller workspace.  Sorted values, permutations, rank means,
Omega and c* must be bit-identical to cutoff_select's on the same input, on two calls in a row of
which the second is smaller (so the array still holds the first call's sums), and sizes beyond
the array must be refused.
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


def both(api, x, **kw):
    import torch

    xd = torch.from_numpy(x).cuda()
    S, N = x.shape
    ref = api.select_cutoff(xd, want_sorted=True, want_perm=True, **kw)
    srt = torch.full((S, N), -7.0, dtype=torch.float32, device="cuda")
    perm = torch.full((S, N), -7, dtype=torch.int32, device="cuda")
    mean = torch.full((N,), -7.0, dtype=torch.float32, device="cuda")
    omega = torch.full((N,), -7.0, dtype=torch.float32, device="cuda")
    cstar = torch.full((2,), -7, dtype=torch.int32, device="cuda")
    api.cutoff_select_static(xd, kw.get("c_min", 1), kw.get("c_max", N), kw.get("t_floor", 0.0), srt, perm, mean,
                             omega, cstar)
    torch.cuda.synchronize()
    assert torch.equal(srt.view(torch.int32), ref["sorted"].view(torch.int32)), "sorted values"
    assert torch.equal(perm, ref["perm"]), "permutation"
    assert torch.equal(mean.view(torch.int32), ref["mean"].view(torch.int32)), "rank means"
    assert torch.equal(omega.view(torch.int32), ref["omega"].view(torch.int32)), "omega"
    c = cstar.cpu()
    assert (int(c[0]), int(c[1])) == (ref["cstar"], ref["status"])
    # without the optional outputs
    cstar2 = torch.full((2,), -7, dtype=torch.int32, device="cuda")
    api.cutoff_select_static(xd, kw.get("c_min", 1), kw.get("c_max", N), kw.get("t_floor", 0.0), None, None, None,
                             None, cstar2)
    torch.cuda.synchronize()
    assert torch.equal(cstar2, cstar)


def test_two_calls_in_a_row_second_smaller(api):
    big = synth.make_runtime_matrix("lognormal_stragglers", 4099, 512, seed=11)
    small = synth.make_runtime_matrix("normal", 130, 48, seed=12)
    both(api, big)
    both(api, small, t_floor=-np.inf)
    both(api, small[:1, :7].copy(), t_floor=-np.inf)
    both(api, big[:700], c_min=3, c_max=400, t_floor=0.5)


def test_largest_preset_shape_fits(api):
    x = synth.make_runtime_matrix("lognormal_stragglers", 8192, 2048, seed=13)
    assert api.cutoff_select_workspace(8192, 2048) <= api.cutoff_select_static_max_workspace()
    both(api, x)
    both(api, x[:300, :2000].copy())


def test_sizes_beyond_the_array_are_refused(api):
    import torch

    S, N = 8192, 4096
    assert api.cutoff_select_workspace(S, N) > api.cutoff_select_static_max_workspace()
    x = torch.ones((S, N), dtype=torch.float32, device="cuda")
    cstar = torch.full((2,), -7, dtype=torch.int32, device="cuda")
    with pytest.raises(api.DkfError) as e:
        api.cutoff_select_static(x, 1, N, 0.0, None, None, None, None, cstar)
    assert e.value.code == api.DKF_EUNSUPPORTED
    torch.cuda.synchronize()
    assert int(cstar[0]) == -7  # nothing was launched
    with pytest.raises(api.DkfError) as e:
        api.cutoff_select_static(x[:16].contiguous(), 5, 2, 0.0, None, None, None, None, cstar)  # c_min > c_max
    assert e.value.code == api.DKF_EINVAL
