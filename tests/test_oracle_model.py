"""Pins for the oracle's model stages (window, RNN encoders, guide chain,
gated transition, emission) -- CPU only.

The paper prints no numbers for these stages, so they are pinned by weight
settings under which each equation of Sec. 3.1.3 collapses to a closed form
that is written here differently from the oracle's loops (collapsed matrix
products, analytic covariances), plus structural facts (which inputs an
output may depend on).  A float64 numpy transcription is kept as an extra
index check; it is not counted as a pin.
"""
import numpy as np
import pytest

import oracle
import cluster_synth as synth


def custom(N=6, L=4, Z=3, H=5, R=7, S=64, idx=9):
    return synth.ClusterConfig("custom", idx, N, L, Z, H, R, S, "f32", 50, "iid_stragglers_tiny")


def softplus(v):
    return np.logaddexp(0.0, v)


def ready_model(cfg, w, trace=None, act=0):
    m = oracle.OracleModel(cfg, synth.pack_blob(cfg, w), emit_mean_act=act)
    trace = synth.make_trace(cfg) if trace is None else trace
    rc = None
    for t in range(cfg.lag):
        rc = m.filter_step(trace[t])
    assert rc == oracle.OK
    return m, trace


# ---- window and normaliser ------------------------------------------------------

def test_warmup_and_normaliser_constant_trace():
    cfg = custom()
    w = synth.make_weights(cfg)
    m = oracle.OracleModel(cfg, synth.pack_blob(cfg, w))
    a = 3.25
    for t in range(cfg.lag):
        rc = m.filter_step(np.full(cfg.n_workers, a))
        assert rc == (oracle.WARMUP if t < cfg.lag - 1 else oracle.OK)
    assert m.scale == pytest.approx(2 * a)
    # every normalised entry is 0.5: with no recurrence the encoding is ReLU(0.5 rowsum(W) + b)
    w["rnn_f_w_hh"][:] = 0
    m2, _ = ready_model(cfg, w, np.full((cfg.lag, cfg.n_workers), a, dtype=np.float32))
    hl, _ = m2.encode_window()
    expect = np.maximum(0.5 * w["rnn_f_w_ih"].astype(np.float64).sum(1) + w["rnn_f_b_ih"] + w["rnn_f_b_hh"], 0)
    assert np.allclose(hl, np.tile(expect, (cfg.lag, 1)), rtol=1e-12, atol=1e-14)


def test_normaliser_is_fixed_by_the_first_window():
    cfg = custom()
    m, tr = ready_model(cfg, synth.make_weights(cfg))
    s0 = m.scale
    assert s0 == pytest.approx(2 * tr[:cfg.lag].astype(np.float64).mean())
    for t in range(cfg.lag, cfg.lag + 7):
        m.filter_step(tr[t] * 10)
    assert m.scale == s0


def test_bad_observations_are_rejected():
    cfg = custom()
    m = oracle.OracleModel(cfg, synth.make_blob(cfg))
    for bad in [0.0, -1.0, np.nan, np.inf]:
        x = np.ones(cfg.n_workers)
        x[2] = bad
        with pytest.raises(ValueError):
            m.filter_step(x)


def test_window_slides():
    cfg = custom()
    w = synth.make_weights(cfg)
    m, tr = ready_model(cfg, w)
    for t in range(cfg.lag, cfg.lag + 3):
        m.filter_step(tr[t])
    hl, hr = m.encode_window()
    # a fresh model fed only the last L vectors has its own normaliser s'; encodings depend
    # on x / s alone, so dividing its input weights by f = s / s' must reproduce them
    win = tr[3:cfg.lag + 3].astype(np.float64)
    f = m.scale / (2 * win.mean())
    w2 = {k: v.copy() for k, v in w.items()}
    w2["rnn_f_w_ih"] = (w["rnn_f_w_ih"].astype(np.float64) / f).astype(np.float32)
    w2["rnn_b_w_ih"] = (w["rnn_b_w_ih"].astype(np.float64) / f).astype(np.float32)
    m3 = oracle.OracleModel(cfg, synth.pack_blob(cfg, w2))
    for row in win:
        m3.filter_step(row)
    hl3, hr3 = m3.encode_window()
    assert np.allclose(hl, hl3, rtol=1e-6, atol=1e-9) and np.allclose(hr, hr3, rtol=1e-6, atol=1e-9)


# ---- RNN encoders ---------------------------------------------------------------

def test_rnn_single_step_is_one_affine_relu():
    cfg = custom(L=1)
    w = synth.make_weights(cfg)
    m, tr = ready_model(cfg, w)
    xn = tr[0].astype(np.float64) / m.scale
    hl, hr = m.encode_window()
    for d, h in (("f", hl), ("b", hr)):
        e = np.maximum(w[f"rnn_{d}_w_ih"].astype(np.float64) @ xn + w[f"rnn_{d}_b_ih"] + w[f"rnn_{d}_b_hh"], 0)
        assert np.allclose(h[0], e, rtol=1e-13, atol=1e-15)


def test_rnn_directions_and_dependence():
    cfg = custom(L=5)
    w = synth.make_weights(cfg, std=0.4)
    m, tr = ready_model(cfg, w)
    hl, hr = m.encode_window()
    tr2 = tr.copy()
    tr2[0] *= 1.0 + 0.5 * np.arange(cfg.n_workers) / cfg.n_workers  # perturb the oldest vector only
    tr2[0] *= tr[0].sum() / tr2[0].sum()  # keep the window mean, hence the normaliser
    m2, _ = ready_model(cfg, w, tr2)
    assert m2.scale == pytest.approx(m.scale, rel=1e-6)
    hl2, hr2 = m2.encode_window()
    assert not np.allclose(hl2[-1], hl[-1])  # the forward state carries the oldest vector to the end
    assert np.allclose(hr2[1:], hr[1:], rtol=1e-5, atol=1e-7)  # the backward state at t > 0 never sees it
    assert not np.allclose(hr2[0], hr[0])
    # first forward / last backward states have no history
    xn = tr.astype(np.float64) / m.scale
    e0 = np.maximum(w["rnn_f_w_ih"].astype(np.float64) @ xn[0] + w["rnn_f_b_ih"] + w["rnn_f_b_hh"], 0)
    eL = np.maximum(w["rnn_b_w_ih"].astype(np.float64) @ xn[cfg.lag - 1] + w["rnn_b_b_ih"] + w["rnn_b_b_hh"], 0)
    assert np.allclose(hl[0], e0, rtol=1e-12) and np.allclose(hr[-1], eL, rtol=1e-12)


def test_rnn_recurrence_as_matrix_power():
    # non-negative weights and inputs keep every ReLU inactive: the RNN is then linear,
    # hl_t = sum_i A^i (B x_{t-i} + b), written here with explicit matrix powers
    cfg = custom(L=4)
    w = {k: np.abs(v) for k, v in synth.make_weights(cfg, std=0.3).items()}
    m, tr = ready_model(cfg, w)
    xn = tr[:cfg.lag].astype(np.float64) / m.scale
    hl, hr = m.encode_window()
    for d, h, order in (("f", hl, range(cfg.lag)), ("b", hr, range(cfg.lag - 1, -1, -1))):
        A = w[f"rnn_{d}_w_hh"].astype(np.float64)
        B = w[f"rnn_{d}_w_ih"].astype(np.float64)
        b = w[f"rnn_{d}_b_ih"].astype(np.float64) + w[f"rnn_{d}_b_hh"]
        seen = []
        for t in order:
            seen.insert(0, t)
            e = sum(np.linalg.matrix_power(A, i) @ (B @ xn[u] + b) for i, u in enumerate(seen))
            assert np.allclose(h[t], e, rtol=1e-11)


# ---- guide chain ------------------------------------------------------------------

def test_guide_combiner_thirds_and_last_step_noise():
    cfg = custom(L=3)
    w = synth.make_weights(cfg, std=0.3)
    w["comb_w"][:] = 0
    w["comb_b"][:] = 0  # tanh(0) = 0: h_out = (h_left + h_right)/3
    w["sig_w"][:] = 0   # sigma_q = softplus(b)
    m, _ = ready_model(cfg, w)
    hl, hr = m.encode_window()
    eq, ez, ex = synth.make_noise(cfg)
    _, st = m.sample_runtimes(eq, ez, ex, stages=True)
    mu = w["mu_w"].astype(np.float64) @ ((hl[-1] + hr[-1]) / 3) + w["mu_b"]
    expect = mu[None, :] + softplus(w["sig_b"].astype(np.float64))[None, :] * eq[-1].astype(np.float64)
    assert np.allclose(st["z_T"], expect, rtol=1e-12, atol=1e-14)
    # saturated combiner: tanh -> 1
    w["comb_b"][:] = 30.0
    m2, _ = ready_model(cfg, w)
    _, st2 = m2.sample_runtimes(eq, ez, ex, stages=True)
    mu2 = w["mu_w"].astype(np.float64) @ ((1 + hl[-1] + hr[-1]) / 3) + w["mu_b"]
    assert np.allclose(st2["z_T"] - expect, (mu2 - mu)[None, :], rtol=1e-9, atol=1e-12)


def test_guide_scale_is_computed_from_the_mean():
    cfg = custom(L=1)
    w = synth.make_weights(cfg, std=0.3)
    w["comb_w"][:] = 0
    m, _ = ready_model(cfg, w)
    hl, hr = m.encode_window()
    eq, ez, ex = synth.make_noise(cfg)
    _, st = m.sample_runtimes(eq, ez, ex, stages=True)
    h_out = (np.tanh(w["comb_b"].astype(np.float64)) + hl[0] + hr[0]) / 3
    mu = w["mu_w"].astype(np.float64) @ h_out + w["mu_b"]
    sig = softplus(w["sig_w"].astype(np.float64) @ mu + w["sig_b"])
    assert np.allclose(st["z_T"], mu + sig * eq[0].astype(np.float64), rtol=1e-12)


def test_guide_chain_feeds_previous_latent_and_z0():
    cfg = custom(L=2)
    w = synth.make_weights(cfg, std=0.5)
    m, _ = ready_model(cfg, w)
    eq, ez, ex = synth.make_noise(cfg)
    _, a = m.sample_runtimes(eq, ez, ex, stages=True)
    eq2 = eq.copy()
    eq2[0, 5] += 1.0  # first-step noise of sample 5 only
    _, b = m.sample_runtimes(eq2, ez, ex, stages=True)
    changed = np.any(a["z_T"] != b["z_T"], axis=1)
    assert changed[5] and changed.sum() == 1
    w2 = dict(w)
    w2["z0"] = w["z0"] + 1.0
    m2, _ = ready_model(cfg, w2)
    _, c = m2.sample_runtimes(eq, ez, ex, stages=True)
    assert np.all(np.any(a["z_T"] != c["z_T"], axis=1))


# ---- transition and emission ---------------------------------------------------------

def linear_gaussian_weights(cfg, gate_bias):
    w = synth.make_weights(cfg, std=0.4)
    w["comb_w"][:] = 0
    w["mu_w"][:] = 0      # mu_q = b_mu
    w["gate2_w"][:] = 0
    w["gate2_b"][:] = gate_bias
    w["tscale_w"][:] = 0  # H = softplus(b)
    w["escale2_w"][:] = 0  # J = softplus(b)
    return w


def test_gate_closed_gives_linear_gaussian_state_space():
    cfg = custom(S=4000)
    w = linear_gaussian_weights(cfg, -60.0)
    m, _ = ready_model(cfg, w)
    eq, ez, ex = synth.make_noise(cfg)
    x, st = m.sample_runtimes(eq, ez, ex, stages=True)
    d = {k: v.astype(np.float64) for k, v in w.items()}
    sig_q = softplus(d["sig_w"] @ d["mu_b"] + d["sig_b"])
    zT = d["mu_b"] + sig_q * eq[-1]
    zn = zT @ d["lin_w"].T + d["lin_b"] + softplus(d["tscale_b"]) * ez
    A = d["emean2_w"] @ d["emean1_w"]  # the two identity layers of I collapse to one matrix
    a0 = d["emean2_w"] @ d["emean1_b"] + d["emean2_b"]
    mean = zn @ A.T + a0
    xs = m.scale * (mean + softplus(d["escale2_b"]) * ex)
    assert np.allclose(st["z_next"], zn, rtol=1e-10, atol=1e-12)
    assert np.allclose(st["emit_mean"], mean, rtol=1e-10, atol=1e-12)
    assert np.allclose(x, xs, rtol=1e-10, atol=1e-12)
    # analytic first and second moments of x (in units of s)
    cov_z = np.diag(sig_q ** 2)
    cov_zn = d["lin_w"] @ cov_z @ d["lin_w"].T + np.diag(softplus(d["tscale_b"]) ** 2)
    cov_x = A @ cov_zn @ A.T + np.diag(softplus(d["escale2_b"]) ** 2)
    mean_x = A @ (d["lin_w"] @ d["mu_b"] + d["lin_b"]) + a0
    xs_n = x / m.scale
    se = np.sqrt(np.diag(cov_x) / cfg.samples)
    assert np.all(np.abs(xs_n.mean(0) - mean_x) < 5 * se)
    emp = np.cov(xs_n.T)
    assert np.allclose(emp, cov_x, atol=6 * np.abs(cov_x).max() / np.sqrt(cfg.samples))


def test_gate_open_gives_the_proposed_mean():
    cfg = custom()
    w = linear_gaussian_weights(cfg, +60.0)
    m, _ = ready_model(cfg, w)
    eq, ez, ex = synth.make_noise(cfg)
    _, st = m.sample_runtimes(eq, ez, ex, stages=True)
    d = {k: v.astype(np.float64) for k, v in w.items()}
    zT = st["z_T"]
    h = np.maximum(zT @ d["prop1_w"].T + d["prop1_b"], 0) @ d["prop2_w"].T + d["prop2_b"]
    assert np.allclose(st["z_next"], h + softplus(d["tscale_b"]) * ez, rtol=1e-10, atol=1e-12)


def test_half_open_gate_and_transition_scale():
    cfg = custom()
    w = synth.make_weights(cfg, std=0.4)
    w["gate2_w"][:] = 0
    w["gate2_b"][:] = 0  # g = 1/2 exactly
    m, _ = ready_model(cfg, w)
    eq, ez, ex = synth.make_noise(cfg)
    _, st = m.sample_runtimes(eq, ez, ex, stages=True)
    d = {k: v.astype(np.float64) for k, v in w.items()}
    zT = st["z_T"]
    h = np.maximum(zT @ d["prop1_w"].T + d["prop1_b"], 0) @ d["prop2_w"].T + d["prop2_b"]
    G = 0.5 * (zT @ d["lin_w"].T + d["lin_b"]) + 0.5 * h
    Hs = softplus(np.maximum(G, 0) @ d["tscale_w"].T + d["tscale_b"])
    assert np.allclose(st["z_next"], G + Hs * ez, rtol=1e-10, atol=1e-12)


def test_all_zero_matrices_emit_iid_gaussians():
    cfg = custom(S=512)
    w = synth.make_weights(cfg)
    for k in w:
        if k.endswith("_w"):
            w[k][:] = 0
    m, _ = ready_model(cfg, w)
    eq, ez, ex = synth.make_noise(cfg)
    x = m.sample_runtimes(eq, ez, ex)
    expect = m.scale * (w["emean2_b"].astype(np.float64) + softplus(w["escale2_b"].astype(np.float64)) * ex)
    assert np.allclose(x, expect, rtol=1e-12, atol=1e-14)


def test_emission_scale_is_fed_by_the_mean_and_activation_switch():
    cfg = custom()
    w = synth.make_weights(cfg, std=0.5)
    eq, ez, ex = synth.make_noise(cfg)
    d = {k: v.astype(np.float64) for k, v in w.items()}
    for act in (0, 1):
        m, _ = ready_model(cfg, w, act=act)
        _, st = m.sample_runtimes(eq, ez, ex, stages=True)
        hid = st["z_next"] @ d["emean1_w"].T + d["emean1_b"]
        if act:
            hid = np.maximum(hid, 0)
        mean = hid @ d["emean2_w"].T + d["emean2_b"]
        sd = softplus(np.maximum(mean @ d["escale1_w"].T + d["escale1_b"], 0) @ d["escale2_w"].T + d["escale2_b"])
        assert np.allclose(st["emit_mean"], mean, rtol=1e-10, atol=1e-12)
        assert np.allclose(st["emit_sd"], sd, rtol=1e-10, atol=1e-12)


def test_zero_noise_rows_are_identical_and_rows_subset():
    cfg = custom()
    m, _ = ready_model(cfg, synth.make_weights(cfg, std=0.4))
    eq, ez, ex = synth.make_noise(cfg)
    x0 = m.sample_runtimes(0 * eq, 0 * ez, 0 * ex)
    assert np.all(x0 == x0[0])
    x = m.sample_runtimes(eq, ez, ex)
    rows = np.array([5, 0, 63, 17], dtype=np.int32)
    assert np.array_equal(m.sample_runtimes(eq, ez, ex, rows=rows), x[rows])


def test_trace_scaling_scales_samples_and_keeps_the_cutoff():
    cfg = synth.CONFIGS["tiny"]
    w = synth.make_weights(cfg)
    tr = synth.make_trace(cfg)
    eq, ez, ex = synth.make_noise(cfg)
    m1, _ = ready_model(cfg, w, tr)
    m2, _ = ready_model(cfg, w, tr * np.float32(8.0))
    x1, x2 = m1.sample_runtimes(eq, ez, ex), m2.sample_runtimes(eq, ez, ex)
    assert np.allclose(x2, 8.0 * x1, rtol=1e-9)
    assert m1.predict_cutoff(eq, ez, ex) == m2.predict_cutoff(eq, ez, ex)


# ---- extra: float64 numpy transcription (index check, not a pin) ----------------------

def numpy_pipeline(cfg, w, window, s, eq, ez, ex, act=0):
    d = {k: v.astype(np.float64) for k, v in w.items()}
    xn = window.astype(np.float64) / s
    L, R = cfg.lag, cfg.rnn_dim
    hl, hr = np.zeros((L, R)), np.zeros((L, R))
    h = np.zeros(R)
    for t in range(L):
        h = np.maximum(d["rnn_f_w_ih"] @ xn[t] + d["rnn_f_b_ih"] + d["rnn_f_w_hh"] @ h + d["rnn_f_b_hh"], 0)
        hl[t] = h
    h = np.zeros(R)
    for t in reversed(range(L)):
        h = np.maximum(d["rnn_b_w_ih"] @ xn[t] + d["rnn_b_b_ih"] + d["rnn_b_w_hh"] @ h + d["rnn_b_b_hh"], 0)
        hr[t] = h
    z = np.tile(d["z0"], (eq.shape[1], 1))
    for t in range(L):
        ho = (np.tanh(z @ d["comb_w"].T + d["comb_b"]) + hl[t] + hr[t]) / 3
        mu = ho @ d["mu_w"].T + d["mu_b"]
        z = mu + softplus(mu @ d["sig_w"].T + d["sig_b"]) * eq[t]
    g = 1 / (1 + np.exp(-(np.maximum(z @ d["gate1_w"].T + d["gate1_b"], 0) @ d["gate2_w"].T + d["gate2_b"])))
    hh = np.maximum(z @ d["prop1_w"].T + d["prop1_b"], 0) @ d["prop2_w"].T + d["prop2_b"]
    G = (1 - g) * (z @ d["lin_w"].T + d["lin_b"]) + g * hh
    zn = G + softplus(np.maximum(G, 0) @ d["tscale_w"].T + d["tscale_b"]) * ez
    hid = zn @ d["emean1_w"].T + d["emean1_b"]
    if act:
        hid = np.maximum(hid, 0)
    mean = hid @ d["emean2_w"].T + d["emean2_b"]
    sd = softplus(np.maximum(mean @ d["escale1_w"].T + d["escale1_b"], 0) @ d["escale2_w"].T + d["escale2_b"])
    return s * (mean + sd * ex)


@pytest.mark.parametrize("name,S", [("tiny", 256), ("medium", 64)])
def test_numpy_transcription_agrees(name, S):
    cfg = synth.CONFIGS[name].with_samples(S)
    w = synth.make_weights(cfg)
    m, tr = ready_model(cfg, w)
    eq, ez, ex = synth.make_noise(cfg)
    s_first = 2 * tr[:cfg.lag].astype(np.float64).mean()
    x0 = m.sample_runtimes(eq, ez, ex)
    assert np.allclose(x0, numpy_pipeline(cfg, w, tr[:cfg.lag], s_first, eq, ez, ex), rtol=1e-9, atol=1e-11)
    for t in range(cfg.lag, cfg.lag + 3):
        m.filter_step(tr[t])
    x3 = m.sample_runtimes(eq, ez, ex)
    assert np.allclose(x3, numpy_pipeline(cfg, w, tr[3:cfg.lag + 3], s_first, eq, ez, ex), rtol=1e-9, atol=1e-11)
