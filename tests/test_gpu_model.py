"""GPU parity: filtering, guide trajectories, transition and emission against the CPU oracle.

Both sides get identical seeded weights, traces and Gaussian noise tensors.
fp32 path tolerance: 1e-4 relative to max(|ref|, rms(ref)) per tensor (the
kernels accumulate dot products of up to a few thousand terms in fp32 through
about 4 L + 10 dependent layers; the oracle is fp64).
"""
import numpy as np
import pytest

import oracle
import cluster_synth as synth
from gpu_util import cstar_in_tie_band, rel_err

pytestmark = pytest.mark.gpu
TOL = 1e-4


@pytest.fixture(scope="module")
def api():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1803_04209_amd import api

    return api


def cuda(*arrays):
    import torch

    return [torch.from_numpy(np.ascontiguousarray(a)).cuda() for a in arrays]


# kernel variants of the sampling stage (dkf_set_sampler): every one must meet the same tolerance
WAVE16, WAVE4, STAGED, SPLIT = 1, 2, 3, 4


def make_pair(api, cfg, weights=None, act=0, pushes=None, std=0.1, mlp_dtype=None, sampler=0):
    w = synth.make_weights(cfg, std) if weights is None else weights
    blob = synth.pack_blob(cfg, w)
    g = api.Predictor(cfg, blob, emit_mean_act=act, mlp_dtype=mlp_dtype)
    g.set_sampler(sampler)
    o = oracle.OracleModel(cfg, blob, emit_mean_act=act)
    tr = synth.make_trace(cfg)
    n = cfg.lag if pushes is None else pushes
    for t in range(n):
        rg = g.filter_step(tr[t])
        ro = o.filter_step(tr[t])
        assert rg == ro
    return g, o, tr


def compare_stages(api, cfg, g, o, S=None, rows=None, tol=TOL):
    eq, ez, ex = synth.make_noise(cfg, S)
    deq, dez, dex = cuda(eq, ez, ex)
    x, st = g.sample_runtimes(deq, dez, dex, stages=True)
    xo, so = o.sample_runtimes(eq, ez, ex, rows=rows, stages=True)
    sel = slice(None) if rows is None else rows
    hl, hr = o.encode_window()
    errs = {
        "ctx": rel_err(st["ctx"].cpu().numpy(), hl + hr),
        "z_T": rel_err(st["z_T"].cpu().numpy()[sel], so["z_T"]),
        "z_next": rel_err(st["z_next"].cpu().numpy()[sel], so["z_next"]),
        "emit_mean": rel_err(st["emit_mean"].cpu().numpy()[sel], so["emit_mean"]),
        "emit_sd": rel_err(st["emit_sd"].cpu().numpy()[sel], so["emit_sd"]),
        "samples": rel_err(x.cpu().numpy()[sel], xo),
    }
    assert all(e <= tol for e in errs.values()), errs
    # the same call without stage outputs runs the kernels the decision path and the benchmark run
    # (variants without the extra stores; for bf16 whole-tile launches a draw kernel of its own):
    # the same samples up to the order of fp32 additions
    x_plain = g.sample_runtimes(deq, dez, dex)
    plain_err = rel_err(x_plain.cpu().numpy(), x.cpu().numpy().astype(np.float64))
    assert plain_err <= 1e-5, plain_err
    return x, errs


def custom(N=6, L=4, Z=3, H=5, R=7, S=64, idx=9):
    return synth.ClusterConfig("custom", idx, N, L, Z, H, R, S, "f32", 50, "iid_stragglers_tiny")


@pytest.mark.parametrize("cfg", [
    custom(), custom(N=33, L=1, Z=8, H=40, R=36, S=100), custom(N=70, L=7, Z=33, H=65, R=31, S=257),
    custom(N=130, L=3, Z=70, H=129, R=200, S=33), custom(N=40, L=3, Z=8, H=16, R=301, S=32),
    custom(N=24, L=4, Z=8, H=16, R=260, S=32)], ids=["6", "33", "70", "130", "wide-rnn-odd", "wide-rnn"])
@pytest.mark.parametrize("act", [0, 1])
def test_unaligned_sizes_every_stage(api, cfg, act):
    g, o, _ = make_pair(api, cfg, act=act, std=0.3)
    compare_stages(api, cfg, g, o)
    g.close()


@pytest.mark.parametrize("cfg", [
    custom(N=20, L=3, Z=12, H=32, R=32, S=50), custom(N=18, L=2, Z=10, H=31, R=30, S=70),
    custom(N=100, L=4, Z=16, H=128, R=128, S=130), custom(N=1000, L=3, Z=32, H=256, R=256, S=40),
    custom(N=36, L=5, Z=8, H=20, R=24, S=16)], ids=["vec-tail", "scalar", "medium-like", "contended-like", "one-wave"])
@pytest.mark.parametrize("act", [0, 1])
@pytest.mark.parametrize("sampler", [WAVE16, WAVE4, STAGED], ids=["wave16", "wave4", "staged"])
def test_fused_sampler_tails(api, cfg, act, sampler):
    """Sizes that the fused sampler kernels cover, with ragged worker blocks, pad features and partial waves."""
    g, o, _ = make_pair(api, cfg, act=act, std=0.3, sampler=sampler)
    compare_stages(api, cfg, g, o)
    eq, ez, ex = synth.make_noise(cfg)
    x_plain = g.sample_runtimes(*cuda(eq, ez, ex))  # variant without the per-stage outputs
    xo = o.sample_runtimes(eq, ez, ex)
    assert rel_err(x_plain.cpu().numpy(), xo) <= TOL
    g.close()


@pytest.mark.parametrize("cfg", [
    custom(N=100, L=4, Z=16, H=128, R=128, S=130), custom(N=128, L=2, Z=12, H=120, R=113, S=50),
    custom(N=500, L=3, Z=32, H=256, R=256, S=40), custom(N=36, L=5, Z=20, H=250, R=244, S=17),
    custom(N=512, L=2, Z=28, H=241, R=256, S=16), custom(N=4, L=1, Z=4, H=128, R=128, S=1),
    custom(N=1100, L=2, Z=16, H=128, R=128, S=35),
    synth.ClusterConfig("custom", 9, 64, 60, 32, 256, 256, 19, "f32", 70, "iid_stragglers_tiny")],
    ids=["medium-like", "pad-features", "contended-like", "ragged", "full-width", "smallest", "many-workers",
         "long-window"])
@pytest.mark.parametrize("act", [0, 1])
def test_split_sampler_tails(api, cfg, act):
    """The sixteen-samples-per-workgroup kernel: ragged worker blocks (whole wavefronts without a
    block of their own), pad features in every width, a partial last workgroup; a window so long that
    its encodings leave LDS room for four wavefronts' exchange buffers only (the kernel then runs
    with four wavefronts per workgroup instead of eight)."""
    g, o, _ = make_pair(api, cfg, act=act, std=0.3, sampler=SPLIT)
    compare_stages(api, cfg, g, o)
    eq, ez, ex = synth.make_noise(cfg)
    x_plain = g.sample_runtimes(*cuda(eq, ez, ex))  # variant without the per-stage outputs
    xo = o.sample_runtimes(eq, ez, ex)
    assert rel_err(x_plain.cpu().numpy(), xo) <= TOL
    g.close()


def test_tiny_preset_every_decision_position(api):
    cfg = synth.CONFIGS["tiny"]
    g, o, tr = make_pair(api, cfg)
    compare_stages(api, cfg, g, o)
    for t in range(cfg.lag, cfg.lag + 25):
        assert g.filter_step(tr[t]) == o.filter_step(tr[t]) == 0
        if t % 6 == 0:
            compare_stages(api, cfg, g, o)
    g.close()


@pytest.mark.parametrize("sampler", [WAVE16, WAVE4, SPLIT], ids=["wave16", "wave4", "split"])
def test_medium_preset_full_size(api, sampler):
    cfg = synth.CONFIGS["medium"]
    g, o, tr = make_pair(api, cfg, pushes=cfg.lag + 3, sampler=sampler)
    compare_stages(api, cfg, g, o, rows=np.arange(0, cfg.samples, 8, dtype=np.int32))
    g.close()


@pytest.mark.parametrize("name", ["contended", "replay"])
@pytest.mark.parametrize("sampler", [WAVE16, WAVE4, SPLIT], ids=["wave16", "wave4", "split"])
def test_large_fp32_presets_sampled_rows(api, name, sampler):
    cfg = synth.CONFIGS[name]
    g, o, tr = make_pair(api, cfg, pushes=cfg.lag + 2, sampler=sampler)
    rows = np.sort(np.random.default_rng(3).choice(cfg.samples, 192, replace=False)).astype(np.int32)
    rows[0], rows[-1] = 0, cfg.samples - 1
    x, errs = compare_stages(api, cfg, g, o, rows=rows)
    # end to end: the library's cutoff on its own samples equals the oracle's rule on those samples
    res = api.select_cutoff(x)
    ref = oracle.cutoff_select(x.cpu().numpy(), want_sorted=False, want_perm=False)
    assert res["status"] == ref["status"] and cstar_in_tie_band(res["cstar"], ref)
    g.close()


# bf16 matrix inputs (weights and activations rounded to nearest even), fp32 accumulation, against
# the fp64 oracle with unrounded weights: 2e-2 relative to max(|ref|, rms(ref)).
TOL_BF16 = 2e-2


@pytest.mark.parametrize("cfg", [
    custom(), custom(N=33, L=1, Z=8, H=40, R=36, S=100), custom(N=70, L=7, Z=33, H=65, R=31, S=257),
    custom(N=130, L=3, Z=70, H=129, R=200, S=33), custom(N=128, L=10, Z=16, H=128, R=128, S=300),
    custom(N=64, L=4, Z=20, H=200, R=250, S=100), custom(N=40, L=3, Z=64, H=300, R=512, S=41)],
    ids=["6", "33", "70", "130", "medium-like", "quarter-256", "quarter-512"])
@pytest.mark.parametrize("act", [0, 1])
@pytest.mark.parametrize("sampler", [0, STAGED], ids=["auto", "staged"])
def test_bf16_every_stage(api, cfg, act, sampler):
    """auto: the register-resident guide/transition kernel where the sizes allow it (latent <= 64 and a
    multiple of 4, hidden widths <= 512), else the staged one; staged: always the latter."""
    # the presets' weight scale, except for the 512-wide encoder, whose recurrence amplifies at that
    # scale (see the large preset's tests below)
    std = 0.06 if cfg.rnn_dim >= 512 else 0.1
    g, o, _ = make_pair(api, cfg, act=act, std=std, mlp_dtype=api.DKF_DTYPE_BF16, sampler=sampler)
    _, errs = compare_stages(api, cfg, g, o, tol=TOL_BF16)
    print("bf16 stage errors", {k: f"{v:.1e}" for k, v in errs.items()})
    assert errs["ctx"] <= TOL  # the RNN encoders stay fp32
    assert max(errs.values()) > 1e-5  # the bf16 path really ran
    g.close()


@pytest.mark.parametrize("cfg", [
    custom(N=128, L=10, Z=16, H=128, R=128, S=300), custom(N=64, L=4, Z=20, H=200, R=250, S=100),
    custom(N=40, L=3, Z=64, H=300, R=512, S=41), custom(N=2175, L=2, Z=16, H=128, R=128, S=5603)],
    ids=["medium-like", "quarter-256", "quarter-512", "2175"])
@pytest.mark.parametrize("act", [0, 1])
def test_bf16_matches_the_mixed_precision_oracle(api, cfg, act):
    """Against the oracle's own mixed-precision mode (matrices and their inputs rounded to bf16 at
    the same points, sums in fp64) the register-resident bf16 kernels must stay within half the
    bf16 tolerance in the max norm (measured: 1e-3 .. 8e-3).  What is left is fp32 against fp64
    summation and the hardware's exp2/log2: differences of 1e-7 that now and then move a value
    across a bf16 rounding boundary, after which the two sides differ by a whole bf16 step there."""
    std = 0.06 if cfg.rnn_dim >= 512 else 0.1
    w = synth.make_weights(cfg, std)
    blob = synth.pack_blob(cfg, w)
    g = api.Predictor(cfg, blob, emit_mean_act=act, mlp_dtype=api.DKF_DTYPE_BF16)
    o = oracle.OracleModel(cfg, blob, emit_mean_act=act, mlp_bf16=True)
    tr = synth.make_trace(cfg)
    for t in range(cfg.lag):
        g.filter_step(tr[t])
        o.filter_step(tr[t])
    rows = None if cfg.samples <= 512 else np.arange(0, cfg.samples, 37, dtype=np.int32)
    _, errs = compare_stages(api, cfg, g, o, rows=rows, tol=TOL_BF16 / 2)
    print("bf16 kernel vs mixed-precision oracle", {k: f"{v:.1e}" for k, v in errs.items()})
    g.close()


@pytest.mark.parametrize("N,S", [(128, 256), (384, 1024), (256, 300), (200, 512)],
                         ids=["one-tile", "several-tiles", "ragged-samples", "ragged-workers"])
def test_bf16_draw_without_stage_outputs(api, N, S):
    """A launch made of whole tiles that asks for no stage outputs takes a draw kernel of its own
    (the mean's product is accumulated on top of bias + scale * noise): its samples against the
    oracle, and against the kernel that also writes the mean and the scale."""
    cfg = custom(N=N, L=3, Z=16, H=128, R=128, S=S)
    g, o, _ = make_pair(api, cfg, std=0.08, mlp_dtype=api.DKF_DTYPE_BF16)
    eq, ez, ex = synth.make_noise(cfg)
    deq, dez, dex = cuda(eq, ez, ex)
    x_plain = g.sample_runtimes(deq, dez, dex)
    x_staged, _ = g.sample_runtimes(deq, dez, dex, stages=True)
    xo = o.sample_runtimes(eq, ez, ex)
    assert rel_err(x_plain.cpu().numpy(), xo) <= TOL_BF16
    # same operands, same roundings; only the order of the fp32 additions differs
    assert rel_err(x_plain.cpu().numpy(), x_staged.cpu().numpy().astype(np.float64)) <= 1e-5
    g.close()


def test_bf16_2175_workers_ragged_wide_tiles(api):
    """The paper's larger cluster size (2175 workers: not a multiple of anything), enough samples for
    the N-wide emission layers to take their 256-feature tiling, ragged last sample tile."""
    cfg = custom(N=2175, L=2, Z=16, H=128, R=128, S=5603)
    g, o, _ = make_pair(api, cfg, std=0.05, mlp_dtype=api.DKF_DTYPE_BF16)
    rows = np.sort(np.random.default_rng(7).choice(cfg.samples, 48, replace=False)).astype(np.int32)
    rows[0], rows[-1] = 0, cfg.samples - 1
    x, errs = compare_stages(api, cfg, g, o, rows=rows, tol=TOL_BF16)
    print("bf16 N=2175 stage errors", {k: f"{v:.1e}" for k, v in errs.items()})
    res = api.select_cutoff(x)
    ref = oracle.cutoff_select(x.cpu().numpy(), want_sorted=False, want_perm=False)
    assert res["status"] == ref["status"] and cstar_in_tie_band(res["cstar"], ref)
    g.close()


def elementwise_rel(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    rms = np.sqrt(np.mean(ref ** 2))
    return np.abs(np.asarray(got, dtype=np.float64) - ref) / np.maximum(np.abs(ref), rms)


def test_large_bf16_preset_damped_weights_sampled_rows(api):
    """Full size of the large preset with weights N(0, 0.03^2): activations stay O(1) and every
    stage meets 2e-2 in the max norm."""
    cfg = synth.CONFIGS["large_bf16"]
    g, o, tr = make_pair(api, cfg, pushes=cfg.lag + 1, std=0.03)
    rows = np.sort(np.random.default_rng(4).choice(cfg.samples, 96, replace=False)).astype(np.int32)
    rows[0], rows[-1] = 0, cfg.samples - 1
    x, errs = compare_stages(api, cfg, g, o, rows=rows, tol=TOL_BF16)
    print("large_bf16 (std 0.03) stage errors", {k: f"{v:.1e}" for k, v in errs.items()})
    res = api.select_cutoff(x)
    ref = oracle.cutoff_select(x.cpu().numpy(), want_sorted=False, want_perm=False)
    assert res["status"] == ref["status"] and cstar_in_tie_band(res["cstar"], ref)
    g.close()


QUANTILES = (0.5, 0.9, 0.99, 0.999, 0.9999)


def test_large_bf16_preset_raw_weights(api):
    """The preset as specified (every tensor N(0, 0.1^2)) is ill-conditioned: with R = 512 the ReLU
    recurrences grow about 2.6x in variance per step, activations reach 1e5..1e7, the gate's sigmoid
    is a hard switch and every layer amplifies what the one before it rounded away.  The mixed
    precision the preset prescribes is then itself a few 1e-2 away from exact arithmetic, whoever
    implements it.  What is held here:
      * the guide's output z_T meets 2e-2 in the max norm against the fp64 oracle;
      * after the gate, the kernel's error against the fp64 oracle is distributed like the error of
        the oracle's own mixed-precision mode (same rounding points, fp64 sums) against fp64:
        every quantile up to 99.99 % and the share of elements beyond 2e-2 stay within a factor
        1.15 (+1e-4) of the oracle's own, per tensor (measured: within 3 %);
      * the same weights at the same size with fp32 MLPs meet 1e-4 in the max norm
        (test_large_preset_raw_weights_fp32), so nothing but the prescribed rounding is at work."""
    cfg = synth.CONFIGS["large_bf16"]
    g, o, tr = make_pair(api, cfg, pushes=cfg.lag + 1)
    ob = oracle.OracleModel(cfg, synth.make_blob(cfg), mlp_bf16=True)
    for t in range(cfg.lag + 1):
        ob.filter_step(tr[t])
    rows = np.arange(0, cfg.samples, 8, dtype=np.int32)
    eq, ez, ex = synth.make_noise(cfg)
    x, st = g.sample_runtimes(*cuda(eq, ez, ex), stages=True)
    xo, so = o.sample_runtimes(eq, ez, ex, rows=rows, stages=True)
    xb, sb = ob.sample_runtimes(eq, ez, ex, rows=rows, stages=True)
    assert rel_err(st["z_T"].cpu().numpy()[rows], so["z_T"]) <= TOL_BF16
    assert rel_err(sb["z_T"], so["z_T"]) <= TOL_BF16
    so["x"], st["x"], sb["x"] = xo, x, xb
    for k in ("z_next", "emit_mean", "emit_sd", "x"):
        e_gpu = elementwise_rel(st[k].cpu().numpy()[rows], so[k]).ravel()
        e_ref = elementwise_rel(sb[k], so[k]).ravel()
        qg, qr = np.quantile(e_gpu, QUANTILES), np.quantile(e_ref, QUANTILES)
        share_g, share_r = np.mean(e_gpu > TOL_BF16), np.mean(e_ref > TOL_BF16)
        print(f"large_bf16 raw {k}: quantiles kernel {np.array2string(qg, precision=4)} mixed-precision oracle "
              f"{np.array2string(qr, precision=4)}; share beyond 2e-2: {share_g:.4f} vs {share_r:.4f}")
        assert np.all(qg <= 1.15 * qr + 1e-4), (k, qg, qr)
        assert share_g <= 1.15 * share_r + 1e-4, (k, share_g, share_r)
    assert torch_isfinite(x)
    res = api.select_cutoff(x)
    ref = oracle.cutoff_select(x.cpu().numpy(), want_sorted=False, want_perm=False)
    assert res["status"] == ref["status"] and cstar_in_tie_band(res["cstar"], ref)
    g.close()


def test_large_preset_raw_weights_fp32(api):
    """The large preset's sizes and raw weights with fp32 MLPs: every stage within 1e-4 of the
    fp64 oracle in the max norm, on 1024 sampled rows of the full-size launch."""
    cfg = synth.CONFIGS["large_bf16"]
    g, o, _ = make_pair(api, cfg, pushes=cfg.lag + 1, mlp_dtype=api.DKF_DTYPE_F32)
    rows = np.arange(0, cfg.samples, 8, dtype=np.int32)
    _, errs = compare_stages(api, cfg, g, o, rows=rows, tol=TOL)
    print("large preset, fp32 MLPs, raw weights:", {k: f"{v:.1e}" for k, v in errs.items()})
    g.close()


@pytest.mark.parametrize("name", ["tiny", "medium", "replay", "large_bf16"])
def test_calibrated_weights(api, name):
    """Emission biases shifted so that predictions sit where normalised run-times do (mean 0.5, small
    spread): few samples are negative, so nearly every rank is eligible in the cutoff rule."""
    cfg = synth.CONFIGS[name]
    bf16 = cfg.mlp_dtype == "bf16"
    std = 0.03 if bf16 else 0.1   # the large preset's recurrences amplify at 0.1 (see its own tests)
    g, o, _ = make_pair(api, cfg, weights=synth.make_weights(cfg, std, calibrated=True), pushes=cfg.lag + 1)
    rows = np.arange(0, cfg.samples, max(1, cfg.samples // 256), dtype=np.int32)
    x, errs = compare_stages(api, cfg, g, o, rows=rows, tol=TOL_BF16 if bf16 else TOL)
    res = api.select_cutoff(x)
    ref = oracle.cutoff_select(x.cpu().numpy(), want_sorted=False, want_perm=False)
    assert res["status"] == ref["status"] == api.DKF_OK and cstar_in_tie_band(res["cstar"], ref)
    assert np.isfinite(ref["omega"]).sum() >= 0.5 * cfg.n_workers
    g.close()


def torch_isfinite(t):
    import torch

    return bool(torch.isfinite(t).all())


@pytest.mark.parametrize("name", ["tiny", "medium", "odd", "bf16"])
def test_builtin_noise_matches_the_oracle_stream(api, name):
    """No noise tensors: the library draws Philox4x32-10 / Box-Muller normals from the seed; the
    oracle is fed the same stream from its own implementation of the published generator."""
    bf16 = name == "bf16"
    cfg = (custom(N=18, L=2, Z=10, H=31, R=30, S=70) if name == "odd" else
           custom(N=64, L=3, Z=16, H=128, R=128, S=100) if bf16 else synth.CONFIGS[name])
    tol = TOL_BF16 if bf16 else TOL
    g, o, tr = make_pair(api, cfg, pushes=cfg.lag + 2, mlp_dtype=api.DKF_DTYPE_BF16 if bf16 else None)
    for seed in (0, 0x1234_5678_9ABC_DEF0):
        x, st = g.sample_runtimes(S=cfg.samples, seed=seed, stages=True)
        eq, ez, ex = oracle.make_noise(cfg, seed)
        xo, so = o.sample_runtimes(eq, ez, ex, stages=True)
        assert rel_err(st["z_T"].cpu().numpy(), so["z_T"]) <= tol
        assert rel_err(st["emit_mean"].cpu().numpy(), so["emit_mean"]) <= tol
        assert rel_err(x.cpu().numpy(), xo) <= tol
    x2 = g.sample_runtimes(S=cfg.samples, seed=1)
    assert not np.allclose(x2.cpu().numpy(), x.cpu().numpy())
    g.close()


def test_decide_with_builtin_noise(api):
    import torch

    cfg = synth.CONFIGS["tiny"]
    blob = synth.make_blob(cfg)
    tr = synth.make_trace(cfg)
    S = cfg.samples
    graph, eager = api.Predictor(cfg, blob), api.Predictor(cfg, blob)
    for t in range(cfg.lag + 8):
        seed = 1000 + t
        c, status = graph.decide(tr[t], S, seed=seed)
        re = eager.filter_step(tr[t])
        if t < cfg.lag - 1:
            assert status == api.DKF_WARMUP == re
            continue
        x = eager.sample_runtimes(S=S, seed=seed)
        res = api.select_cutoff(x)
        assert (c, status) == (res["cstar"], res["status"])
        assert torch.equal(graph.decide_samples(S), x)
    graph.close()
    eager.close()


def test_warmup_errors_and_reset(api):
    import torch

    cfg = synth.CONFIGS["tiny"]
    blob = synth.make_blob(cfg)
    g = api.Predictor(cfg, blob)
    tr = synth.make_trace(cfg)
    eq, ez, ex = cuda(*synth.make_noise(cfg))
    out = torch.empty((cfg.samples, cfg.n_workers), device="cuda")
    for t in range(cfg.lag - 1):
        assert g.filter_step(tr[t]) == api.DKF_WARMUP
        with pytest.raises(api.DkfError) as e:
            g.sample_runtimes(eq, ez, ex, out=out)
        assert e.value.code == api.DKF_ENOTREADY
    bad = tr[0].copy()
    bad[3] = -1.0
    with pytest.raises(api.DkfError) as e:
        g.filter_step(bad)
    assert e.value.code == api.DKF_EBADOBS
    assert g.filter_step(tr[cfg.lag - 1]) == api.DKF_OK  # the rejected vector did not enter the window
    a = g.sample_runtimes(eq, ez, ex).clone()
    g.reset()
    assert g.filter_step(tr[0]) == api.DKF_WARMUP
    for t in range(1, cfg.lag):
        g.filter_step(tr[t])
    b = g.sample_runtimes(eq, ez, ex)
    assert torch.equal(a, b)
    with pytest.raises(api.DkfError):
        api.dkf_sample_runtimes(g.handle, cfg.samples + 1, eq, ez, ex, 0, out)
    with pytest.raises(api.DkfError) as e:
        api.dkf_sample_runtimes(g.handle, cfg.samples, eq, None, ex, 0, out)  # some but not all tensors
    assert e.value.code == api.DKF_EINVAL
    with pytest.raises(api.DkfError) as e:
        api.dkf_load_weights(api.make_config(cfg), blob[:-4])
    assert e.value.code == api.DKF_EBLOB
    g.close()


def test_state_roundtrip_resumes_bit_exactly(api):
    import torch

    cfg = synth.CONFIGS["tiny"]
    blob = synth.make_blob(cfg)
    tr = synth.make_trace(cfg)
    eq, ez, ex = cuda(*synth.make_noise(cfg))
    a = api.Predictor(cfg, blob)
    for t in range(cfg.lag + 4):
        a.filter_step(tr[t])
    state = a.get_state()
    b = api.Predictor(cfg, blob)
    b.set_state(state)
    assert torch.equal(a.sample_runtimes(eq, ez, ex), b.sample_runtimes(eq, ez, ex))
    for t in range(cfg.lag + 4, cfg.lag + 9):
        a.filter_step(tr[t])
        b.filter_step(tr[t])
    assert torch.equal(a.sample_runtimes(eq, ez, ex), b.sample_runtimes(eq, ez, ex))
    a.close()
    b.close()


@pytest.mark.parametrize("name", ["tiny", "medium", "contended", "replay", "large_bf16"])
def test_decide_graph_replays_match_eager(api, name):
    """Every replay of the captured decision graph (the path the benchmark times, at the presets' full
    sizes) is checked against the eager calls, and its decision against the oracle's rule."""
    import torch

    cfg = synth.CONFIGS[name]
    blob = synth.make_blob(cfg)
    tr = synth.make_trace(cfg)
    S = cfg.samples
    eq, ez, ex = cuda(*synth.make_noise(cfg))
    graph, eager = api.Predictor(cfg, blob), api.Predictor(cfg, blob)
    # medium and replay: the decision's sampler sorts its own rows, the eager calls sort in cutoff_select
    assert graph.decide_sorts_in_sampler(S) == (name in ("medium", "replay"))
    for t in range(cfg.lag + (12 if cfg.samples * cfg.n_workers <= 1 << 20 else 4)):
        c, status = graph.decide(tr[t], S, eq, ez, ex)
        re = eager.filter_step(tr[t])
        if t < cfg.lag - 1:
            assert status == api.DKF_WARMUP == re and c == cfg.n_workers
            continue
        x = eager.sample_runtimes(eq, ez, ex)
        res = api.select_cutoff(x)
        assert (c, status) == (res["cstar"], res["status"])
        xg = graph.decide_samples(S)
        assert torch.equal(xg, x)
        orc = oracle.cutoff_select(x.cpu().numpy(), want_sorted=False, want_perm=False)
        assert cstar_in_tie_band(c, orc)
        if t % 5 == 0:
            # new noise in the same buffers: replays must read it
            nq, nz, nx = cuda(*synth.make_noise(cfg, draw=t))
            eq.copy_(nq); ez.copy_(nz); ex.copy_(nx)
            torch.cuda.synchronize()
    graph.close()
    eager.close()


@pytest.mark.parametrize("widths", [dict(N=128, Z=16, H=128, R=128), dict(N=512, Z=32, H=256, R=256),
                                    dict(N=128, Z=32, H=256, R=256)])
@pytest.mark.parametrize("S", [16, 272, 1000, 4096])
def test_decide_with_rows_sorted_in_the_sampler(api, widths, S):
    """dkf_decide where the sampler sorts its own rows (S a multiple of 16) and where it cannot
    (S = 1000): the decision equals cutoff_select's on the samples of the eager call, and the
    oracle's rule holds, over several steps with fresh noise."""
    cfg = custom(L=4, S=S, **widths)
    blob = synth.make_blob(cfg, std=0.05)
    tr = synth.make_trace(cfg)
    graph, eager = api.Predictor(cfg, blob), api.Predictor(cfg, blob)
    assert graph.sampler_in_use(S) == SPLIT
    assert graph.decide_sorts_in_sampler(S) == (S % 16 == 0)
    for t in range(cfg.lag + 5):
        eq, ez, ex = cuda(*synth.make_noise(cfg, draw=t))
        c, status = graph.decide(tr[t], S, eq, ez, ex)
        re = eager.filter_step(tr[t])
        if t < cfg.lag - 1:
            assert status == api.DKF_WARMUP == re
            continue
        x = eager.sample_runtimes(eq, ez, ex)
        res = api.select_cutoff(x)
        orc = oracle.cutoff_select(x.cpu().numpy(), want_sorted=False, want_perm=False)
        assert status == res["status"]
        # (the two paths add the rank sums in different orders: equal decisions up to ties in Omega)
        assert c == res["cstar"] or cstar_in_tie_band(c, orc)
        assert cstar_in_tie_band(c, orc)
    with pytest.raises(api.DkfError):
        graph.decide_sorts_in_sampler(0)
    graph.close()
    eager.close()


def test_decide_trace_equals_the_single_calls(api):
    """dkf_decide_trace: the same decisions, statuses and final state as one dkf_decide per row."""
    cfg = synth.CONFIGS["tiny"]
    blob = synth.make_blob(cfg)
    tr = synth.make_trace(cfg)
    S = cfg.samples
    eq, ez, ex = cuda(*synth.make_noise(cfg))
    T = cfg.lag + 20
    one, many = api.Predictor(cfg, blob), api.Predictor(cfg, blob)
    singles = [one.decide(tr[t], S, eq, ez, ex) for t in range(T)]
    c, st, lat = many.decide_trace(tr[:T], S, eq, ez, ex)
    assert [(int(a), int(b)) for a, b in zip(c, st)] == singles
    assert st[:cfg.lag - 1].tolist() == [api.DKF_WARMUP] * (cfg.lag - 1) and np.all(c[:cfg.lag - 1] == cfg.n_workers)
    assert np.all(lat > 0) and np.all(lat < 1e6)
    assert one.get_state() == many.get_state()
    # the library's own noise: seed + t per step
    singles = [one.decide(tr[T + t], S, seed=77 + t) for t in range(6)]
    c, st, _ = many.decide_trace(tr[T:T + 6], S, seed=77)
    assert [(int(a), int(b)) for a, b in zip(c, st)] == singles
    # a bad observation stops the replay with its error; the steps before it have been taken
    bad = tr[T + 6:T + 10].copy()
    bad[2, 0] = -1.0
    with pytest.raises(api.DkfError) as e:
        many.decide_trace(bad, S, eq, ez, ex)
    assert e.value.code == api.DKF_EBADOBS
    for t in range(2):
        one.decide(bad[t], S, eq, ez, ex)
    assert one.get_state() == many.get_state()
    with pytest.raises(api.DkfError):
        many.decide_trace(tr[:0], S, eq, ez, ex)
    one.close()
    many.close()


def test_sampler_in_use_follows_sizes_and_setting(api):
    cfg = synth.CONFIGS["medium"]
    g = api.Predictor(cfg, synth.make_blob(cfg))
    assert [g.sampler_in_use(S) for S in (1, 4096, 4097, 8192, 8193)] == [SPLIT, SPLIT, WAVE4, WAVE4, WAVE16]
    g.set_sampler(WAVE16)
    assert g.sampler_in_use(16) == WAVE16
    g.set_sampler(STAGED)
    assert g.sampler_in_use(16) == STAGED
    with pytest.raises(api.DkfError):
        g.sampler_in_use(0)
    g.close()
    cfg = synth.CONFIGS["tiny"]  # widths the sixteen-per-workgroup kernel is not built for
    g = api.Predictor(cfg, synth.make_blob(cfg))
    assert g.sampler_in_use(cfg.samples) == WAVE4
    g.close()
    cfg = custom(N=64, L=2, Z=16, H=128, R=128, S=64)
    g = api.Predictor(cfg, synth.make_blob(cfg), mlp_dtype=api.DKF_DTYPE_BF16)
    assert g.sampler_in_use(64) == STAGED
    g.close()


def test_sampler_variant_selection(api):
    """A variant the model's sizes rule out is refused and the current one stays."""
    cfg = custom(N=130, L=3, Z=70, H=129, R=200, S=33)  # latent too wide for both fused kernels
    g = api.Predictor(cfg, synth.make_blob(cfg))
    for v in (WAVE16, WAVE4, SPLIT):
        with pytest.raises(api.DkfError):
            g.set_sampler(v)
    g.set_sampler(STAGED)
    with pytest.raises(api.DkfError):
        g.set_sampler(7)
    g.close()
