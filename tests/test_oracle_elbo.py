"""Pins of the ELBO trainer (Sec. 3.1.3, model learning) — CPU only.

(1) Its forward pieces agree with the C oracle's stage outputs on the same weights and noise: two
    independent writings (C loops, torch matrix products) of the same equations.
(2) Linear-Gaussian special cases, where the evidence has a closed form that scipy evaluates:
    with the guide set to the exact posterior the single-sample bound equals log p(x) for every
    noise draw; with another guide the importance-weight identity E_q[exp(ELBO)] = p(x) holds and
    the mean bound lies below log p(x) (two time steps, so the chaining through z_{t-1} counts).
(3) Fitting raises the bound on a synthetic trace and the fitted blob loads into the predictor.
"""
import math
from dataclasses import replace

import numpy as np
import pytest
import torch
from scipy.stats import multivariate_normal

import oracle
from oracle import elbo as E
import cluster_synth as synth


def softplus_inv(y):
    return math.log(math.expm1(y))


@pytest.mark.parametrize("act", [0, 1])
def test_forward_pieces_match_c_oracle(act):
    cfg = synth.CONFIGS["tiny"]
    blob = synth.make_blob(cfg, std=0.3)
    trace = synth.make_trace(cfg)
    m = oracle.OracleModel(cfg, blob, emit_mean_act=act)
    for t in range(cfg.lag + 3):
        m.filter_step(trace[t])
    eps_q, eps_z, eps_x = synth.make_noise(cfg, samples=3)
    _, st = m.sample_runtimes(eps_q, eps_z, eps_x, stages=True)
    hl_c, hr_c = m.encode_window()
    p = E.params_from_blob(cfg, blob, requires_grad=False)
    window = trace[3:3 + cfg.lag].astype(np.float64)
    xhat = torch.tensor(window / m.scale)
    hl, hr = E.encode(p, xhat)
    np.testing.assert_allclose(torch.stack(hl).numpy(), hl_c, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(torch.stack(hr).numpy(), hr_c, rtol=1e-12, atol=1e-13)
    for k in range(3):
        _, zs = E.elbo(p, xhat, torch.tensor(eps_q[:, k].astype(np.float64)), act)
        np.testing.assert_allclose(zs[-1].numpy(), st["z_T"][k], rtol=1e-11, atol=1e-12)
        G, Hs = E.transition(p, zs[-1])
        z_next = G + Hs * torch.tensor(eps_z[k].astype(np.float64))
        np.testing.assert_allclose(z_next.numpy(), st["z_next"][k], rtol=1e-11, atol=1e-12)
        mean, sd = E.emission(p, z_next, act)
        np.testing.assert_allclose(mean.numpy(), st["emit_mean"][k], rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(sd.numpy(), st["emit_sd"][k], rtol=1e-11, atol=1e-12)


def linear_gaussian(L, Js=(0.5, 0.8, 0.6)):
    """Weights that make the model linear-Gaussian: gate shut, constant scales, identity hidden layer."""
    cfg = replace(synth.CONFIGS["tiny"], n_workers=3, lag=L, z_dim=2, hidden=2, rnn_dim=4)
    g = np.random.default_rng(5)
    w = {k: 0.3 * g.standard_normal(s) for k, s in synth.blob_layout(cfg)}
    w["gate2_w"][:] = 0.0
    w["gate2_b"][:] = -60.0          # sigmoid -> 0: G(z) = lin_w z + lin_b
    w["tscale_w"][:] = 0.0           # H(z) = softplus(tscale_b)
    w["tscale_b"] = np.array([softplus_inv(0.7), softplus_inv(1.1)])
    w["emean1_w"] = np.eye(2)
    w["emean1_b"][:] = 0.0
    w["emean2_w"] = np.array([[0.9, 0.0], [0.0, -1.2], [0.6, 0.0]])   # columns with disjoint support
    w["escale2_w"][:] = 0.0          # J(z) = softplus(escale2_b)
    w["escale2_b"] = np.array([softplus_inv(j) for j in Js])
    p = {k: torch.tensor(np.asarray(v, dtype=np.float64)) for k, v in w.items()}
    A = w["emean2_w"] @ w["emean1_w"]
    b = w["emean2_b"]
    F, f = w["lin_w"], w["lin_b"]
    Hs = np.array([0.7, 1.1])
    Js = np.array(Js)
    return cfg, p, A, b, F, f, Hs, Js


def test_single_step_bound_is_tight_at_exact_posterior():
    cfg, p, A, b, F, f, Hs, Js = linear_gaussian(1)
    z0 = p["z0"].numpy()
    m0 = F @ z0 + f                                   # prior mean of z_1
    x = np.array([0.4, -0.3, 1.1])
    evidence = multivariate_normal(A @ m0 + b, A @ np.diag(Hs ** 2) @ A.T + np.diag(Js ** 2)).logpdf(x)
    prec = np.diag(1 / Hs ** 2) + A.T @ np.diag(1 / Js ** 2) @ A
    assert abs(prec[0, 1]) < 1e-15                    # the posterior factorises, as the guide does
    cov = np.linalg.inv(prec)
    mean = cov @ (m0 / Hs ** 2 + A.T @ ((x - b) / Js ** 2))
    p["mu_w"] = torch.zeros_like(p["mu_w"])
    p["mu_b"] = torch.tensor(mean)
    p["sig_w"] = torch.zeros_like(p["sig_w"])
    p["sig_b"] = torch.tensor([softplus_inv(math.sqrt(cov[0, 0])), softplus_inv(math.sqrt(cov[1, 1]))], dtype=E.DT)
    g = torch.Generator().manual_seed(1)
    for _ in range(5):
        eps = torch.randn((1, 2), dtype=torch.float64, generator=g)
        val, _ = E.elbo(p, torch.tensor(x)[None], eps)
        assert abs(float(val) - evidence) < 1e-11
    # any other guide: pointwise, ELBO = log p(x) + log post(z) - log q(z)
    p["mu_b"] = torch.tensor(mean + np.array([0.3, -0.2]))
    p["sig_b"] = torch.tensor([softplus_inv(0.9), softplus_inv(0.4)], dtype=E.DT)
    post = multivariate_normal(mean, cov)
    q = multivariate_normal(mean + np.array([0.3, -0.2]), np.diag([0.9 ** 2, 0.4 ** 2]))
    for _ in range(5):
        eps = torch.randn((1, 2), dtype=torch.float64, generator=g)
        val, zs = E.elbo(p, torch.tensor(x)[None], eps)
        z = zs[0].numpy()
        assert abs(float(val) - (evidence + post.logpdf(z) - q.logpdf(z))) < 1e-11


def test_two_step_importance_identity_and_bound():
    cfg, p, A, b, F, f, Hs, Js = linear_gaussian(2, Js=(2.0, 2.5, 2.2))   # weak observations: the posterior stays near the prior
    z0 = p["z0"].numpy()
    x = np.array([[0.4, -0.3, 1.1], [0.2, 0.5, 0.7]])
    # joint law of (z_1, z_2), then of the stacked observations
    m1 = F @ z0 + f
    P1 = np.diag(Hs ** 2)
    m2 = F @ m1 + f
    P2 = F @ P1 @ F.T + np.diag(Hs ** 2)
    C12 = P1 @ F.T
    mz = np.concatenate([m1, m2])
    Pz = np.block([[P1, C12], [C12.T, P2]])
    AA = np.block([[A, np.zeros_like(A)], [np.zeros_like(A), A]])
    evidence = multivariate_normal(AA @ mz + np.tile(b, 2),
                                   AA @ Pz @ AA.T + np.diag(np.tile(Js ** 2, 2))).logpdf(x.reshape(-1))
    # a guide near the prior, slightly wider, with a small dependence on the encoder states
    p["mu_w"] = 0.05 * p["mu_w"]
    p["mu_b"] = torch.tensor(0.5 * (m1 + m2))
    p["sig_w"] = torch.zeros_like(p["sig_w"])
    p["sig_b"] = torch.tensor([softplus_inv(1.0), softplus_inv(1.5)], dtype=E.DT)
    g = torch.Generator().manual_seed(2)
    n = 6000
    vals = np.empty(n)
    xt = torch.tensor(x)
    for i in range(n):
        vals[i], _ = E.elbo(p, xt, torch.randn((2, 2), dtype=torch.float64, generator=g))
    w = np.exp(vals - evidence)
    se = w.std(ddof=1) / math.sqrt(n)
    assert abs(w.mean() - 1.0) < 4 * se and se < 0.05, (w.mean(), se)
    assert vals.mean() + 4 * vals.std(ddof=1) / math.sqrt(n) < evidence   # Jensen gap is strictly positive here


def test_two_step_bound_pointwise_against_joint_gaussian():
    """ELBO(eps) = log p(x_{1:2}, z_{1:2}) - log q(z_{1:2}), the joint density evaluated as ONE
    10-dimensional Gaussian assembled from the linear model (informative observations)."""
    from scipy.stats import norm

    cfg, p, A, b, F, f, Hs, Js = linear_gaussian(2)
    z0 = p["z0"].numpy()
    x = np.array([[0.4, -0.3, 1.1], [-0.6, 0.5, 0.1]])
    m1 = F @ z0 + f
    P1 = np.diag(Hs ** 2)
    m2 = F @ m1 + f
    P2 = F @ P1 @ F.T + np.diag(Hs ** 2)
    C12 = P1 @ F.T
    mz = np.concatenate([m1, m2])
    Pz = np.block([[P1, C12], [C12.T, P2]])
    AA = np.block([[A, np.zeros_like(A)], [np.zeros_like(A), A]])
    mean = np.concatenate([mz, AA @ mz + np.tile(b, 2)])
    cov = np.block([[Pz, Pz @ AA.T], [AA @ Pz, AA @ Pz @ AA.T + np.diag(np.tile(Js ** 2, 2))]])
    joint = multivariate_normal(mean, cov)
    xt = torch.tensor(x)
    hl, hr = E.encode(p, xt)
    g = torch.Generator().manual_seed(4)
    for _ in range(6):
        val, zs = E.elbo(p, xt, torch.randn((2, 2), dtype=E.DT, generator=g))
        z = [v.numpy() for v in zs]
        logq, prev = 0.0, p["z0"]
        for t in range(2):
            mu, sigma = E.guide_step(p, prev, hl[t], hr[t])
            logq += norm(mu.numpy(), sigma.numpy()).logpdf(z[t]).sum()
            prev = zs[t]
        want = joint.logpdf(np.concatenate([z[0], z[1], x[0], x[1]])) - logq
        assert abs(float(val) - want) < 1e-9


def test_batched_bound_equals_window_by_window():
    cfg = synth.CONFIGS["tiny"]
    p = E.params_from_blob(cfg, synth.make_blob(cfg, std=0.3), requires_grad=False)
    trace = torch.tensor(synth.make_trace(cfg).astype(np.float64))
    g = torch.Generator().manual_seed(7)
    windows = torch.stack([trace[s:s + cfg.lag] for s in (0, 17, 100)])
    eps = torch.randn((3, cfg.lag, cfg.z_dim), dtype=E.DT, generator=g)
    together, _ = E.elbo(p, windows, eps)
    for k in range(3):
        alone, _ = E.elbo(p, windows[k], eps[k])
        assert abs(float(alone) - float(together[k])) < 1e-9 * abs(float(alone))


def test_fit_raises_the_bound_and_the_blob_loads():
    cfg = synth.CONFIGS["tiny"]
    blob = synth.make_blob(cfg)
    trace = synth.make_trace(cfg)
    fitted, hist = E.fit(cfg, blob, trace, steps=120, lr=3e-3, batch=4, seed=3)
    assert np.mean(hist[-20:]) > np.mean(hist[:20]) + 10.0, (np.mean(hist[:20]), np.mean(hist[-20:]))
    assert fitted.shape == blob.shape and fitted.dtype == blob.dtype
    m = oracle.OracleModel(cfg, fitted)
    for t in range(cfg.lag):
        m.filter_step(trace[t])
    eps_q, eps_z, eps_x = synth.make_noise(cfg, samples=64)
    x = m.sample_runtimes(eps_q, eps_z, eps_x)
    assert np.all(np.isfinite(x))
    # same seed, same result: the fit draws every random number from its own generator
    again, _ = E.fit(cfg, blob, trace, steps=3, lr=3e-3, batch=4, seed=3)
    again2, _ = E.fit(cfg, blob, trace, steps=3, lr=3e-3, batch=4, seed=3)
    assert np.array_equal(again, again2)


def test_replay_report_orders_the_comparison_rates():
    """full sync <= best fixed cutoff <= per-step hindsight optimum, and no choice beats hindsight."""
    from oracle import fit_demo

    cfg = synth.CONFIGS["tiny"]
    trace = synth.make_trace(cfg, 60)
    steps, chosen = fit_demo.replay(cfg, synth.make_blob(cfg), trace, first=20, samples=64, stride=3)
    assert steps[0] == 21 and np.all(np.diff(steps) == 3) and steps[-1] <= 59
    r = fit_demo.report(trace, steps, chosen)
    assert r["full_sync"] <= r["best_fixed"] <= r["hindsight"] and r["chosen"] <= r["hindsight"]
    srt = np.sort(trace[steps].astype(np.float64), axis=1)
    assert abs(r["full_sync"] - cfg.n_workers * len(steps) / srt[:, -1].sum()) < 1e-9 * r["full_sync"]
