"""Fitting the run-time model and its inference network by the ELBO (Sec. 3.1.3, "Model Learning
and Amortized Inference"; optimiser: Adam with gradient clipping, Sec. 4.1).

Test infrastructure, not product code: plain PyTorch CPU operations in float64 with autograd,
one statement per equation of the paper.  It exists so that decisions can be examined with
*fitted* weights (the predictor itself is indifferent to where its weights come from); nothing in
the GPU library imports it.

For one fixed-lag window x_{1:L} (already divided by the normaliser) and one reparameterised
trajectory z_{1:L} ~ q_phi the single-sample estimate of the bound is

    ELBO = sum_t [ log p(x_t | z_t) + log p(z_t | z_{t-1}) - log q(z_t | z_{t-1}, x_{1:L}) ]

with the model and guide of Sec. 3.1.3 exactly as the C oracle reads them:
    p(z_t | z_{t-1}) = N(G(z_{t-1}), H(z_{t-1})),  p(x_t | z_t) = N(I(z_t), J(z_t)),
    q(z_t | .) = N(mu, sigma),  mu = K(h_out),  sigma = softplus(L(mu)),
    h_out = (tanh(W_c z_{t-1} + b) + h_left,t + h_right,t) / 3,
the second argument of every N(., .) being a standard deviation.
READING: z_{t-1} at the first window position is the learned vector z0, in the transition density
as in the guide (the same reading as in the predictor).
"""
from __future__ import annotations

import math
from typing import Dict

import numpy as np
import torch
import torch.nn.functional as F

import cluster_synth as synth

DT = torch.float64


def params_from_blob(cfg, blob: np.ndarray, requires_grad: bool = True) -> Dict[str, torch.Tensor]:
    w = synth.unpack_blob(cfg, blob)
    return {k: torch.tensor(v, dtype=DT, requires_grad=requires_grad) for k, v in w.items()}


def blob_from_params(cfg, p: Dict[str, torch.Tensor]) -> np.ndarray:
    return synth.pack_blob(cfg, {k: v.detach().numpy().astype(np.float32) for k, v in p.items()})


def affine(p, name, v):
    """W v + b for one vector, or for every row of a batch [..., n] at once."""
    return F.linear(v, p[name + "_w"], p[name + "_b"])


def encode(p, xhat):
    """h_left,t (forward RNN over x_1..x_t) and h_right,t (backward RNN over x_L..x_t), ReLU cells
    from zero.  xhat is [L][N] or a batch [B][L][N]; returns two lists of L tensors [..., R]."""
    L = xhat.shape[-2]
    hl, hr = [None] * L, [None] * L
    h = torch.zeros(xhat.shape[:-2] + (p["rnn_f_b_ih"].shape[0],), dtype=DT)
    for t in range(L):
        h = torch.relu(F.linear(xhat[..., t, :], p["rnn_f_w_ih"], p["rnn_f_b_ih"])
                       + F.linear(h, p["rnn_f_w_hh"], p["rnn_f_b_hh"]))
        hl[t] = h
    h = torch.zeros_like(h)
    for t in reversed(range(L)):
        h = torch.relu(F.linear(xhat[..., t, :], p["rnn_b_w_ih"], p["rnn_b_b_ih"])
                       + F.linear(h, p["rnn_b_w_hh"], p["rnn_b_b_hh"]))
        hr[t] = h
    return hl, hr


def guide_step(p, z_prev, hl_t, hr_t):
    h_out = (torch.tanh(affine(p, "comb", z_prev)) + hl_t + hr_t) / 3.0
    mu = affine(p, "mu", h_out)
    sigma = F.softplus(affine(p, "sig", mu))
    return mu, sigma


def transition(p, z):
    g = torch.sigmoid(affine(p, "gate2", torch.relu(affine(p, "gate1", z))))
    h = affine(p, "prop2", torch.relu(affine(p, "prop1", z)))
    G = (1.0 - g) * affine(p, "lin", z) + g * h
    Hs = F.softplus(affine(p, "tscale", torch.relu(G)))
    return G, Hs


def emission(p, z, emit_mean_act: int = 0):
    hid = affine(p, "emean1", z)
    if emit_mean_act:
        hid = torch.relu(hid)
    mean = affine(p, "emean2", hid)
    sd = F.softplus(affine(p, "escale2", torch.relu(affine(p, "escale1", mean))))
    return mean, sd


def log_normal(x, mean, sd):
    """log N(x; mean, diag(sd^2)), summed over the last axis."""
    return (-0.5 * ((x - mean) / sd) ** 2 - torch.log(sd) - 0.5 * math.log(2.0 * math.pi)).sum(-1)


def elbo(p, xhat: torch.Tensor, eps: torch.Tensor, emit_mean_act: int = 0):
    """Single-sample ELBO of one window xhat [L][N] for noise eps [L][Z] (or of each window of a
    batch, [B][L][N] and [B][L][Z], giving [B]); also returns z_{1:L}."""
    hl, hr = encode(p, xhat)
    z_prev = p["z0"].expand(xhat.shape[:-2] + p["z0"].shape)
    total = torch.zeros(xhat.shape[:-2], dtype=DT)
    zs = []
    for t in range(xhat.shape[-2]):
        mu, sigma = guide_step(p, z_prev, hl[t], hr[t])
        z = mu + sigma * eps[..., t, :]
        G, Hs = transition(p, z_prev)
        mean, sd = emission(p, z, emit_mean_act)
        total = total + log_normal(xhat[..., t, :], mean, sd) + log_normal(z, G, Hs) - log_normal(z, mu, sigma)
        zs.append(z)
        z_prev = z
    return total, zs


def fit(cfg, blob: np.ndarray, trace: np.ndarray, steps: int, lr: float = 2e-3, clip: float = 10.0,
        batch: int = 8, seed: int = 0, emit_mean_act: int = 0, log=None):
    """Adam with gradient clipping on windows drawn from `trace` [T][N] (seconds).  The normaliser is
    the predictor's: twice the mean of the first window.  Returns (blob, list of mean ELBO per step)."""
    g = torch.Generator().manual_seed(seed)
    p = params_from_blob(cfg, blob)
    opt = torch.optim.Adam(list(p.values()), lr=lr)
    L = cfg.lag
    scale = 2.0 * float(np.mean(trace[:L]))
    xhat_all = torch.tensor(trace / scale, dtype=DT)
    history = []
    for it in range(steps):
        opt.zero_grad()
        starts = torch.randint(0, trace.shape[0] - L + 1, (batch,), generator=g)
        windows = torch.stack([xhat_all[s:s + L] for s in starts.tolist()])
        eps = torch.randn((batch, L, cfg.z_dim), dtype=DT, generator=g)
        loss = -elbo(p, windows, eps, emit_mean_act)[0].mean()
        loss.backward()
        torch.nn.utils.clip_grad_norm_(list(p.values()), clip)
        opt.step()
        history.append(-float(loss.detach()))
        if log and (it % log == 0 or it == steps - 1):
            print(f"step {it:5d}  ELBO per window {history[-1]:12.3f}", flush=True)
    return blob_from_params(cfg, p), history
