#!/usr/bin/env python3
"""Writes tests/golden/scalar_chain.txt: the predictor of Sec. 3.1.3 with every width equal to one
(one worker, one latent, one hidden unit, one RNN unit, one sample), a window of two observations,
worked through as straight-line scalar arithmetic with nothing but `math`.

Every weight, observation and noise value is a multiple of 1/16, hence exact in fp32, so the
numbers written here are the exact-arithmetic answer to double precision.  Two cases: in A every
ReLU that matters is active, in B the gate's hidden unit, the proposed mean's hidden unit, ReLU(G),
the backward RNN's older state and the hidden unit of the emission mean (for its ReLU variant) are
switched off.

Run from the repository root:  python tests/golden/make_scalar_chain.py
It imports nothing of this repository.
"""
import math
from pathlib import Path

CASES = {
    "A": dict(
        x1=1.5, x2=2.5,
        f_w_ih=0.75, f_b_ih=0.125, f_w_hh=0.5, f_b_hh=-0.25,
        b_w_ih=-0.5, b_b_ih=0.875, b_w_hh=0.25, b_b_hh=0.0625,
        comb_w=0.625, comb_b=-0.125, mu_w=1.25, mu_b=0.1875, sig_w=-0.75, sig_b=0.25, z0=0.5,
        gate1_w=1.5, gate1_b=0.25, gate2_w=-0.875, gate2_b=0.5,
        prop1_w=0.75, prop1_b=-0.125, prop2_w=1.125, prop2_b=0.3125,
        lin_w=-0.625, lin_b=0.4375, tscale_w=0.5, tscale_b=-0.375,
        emean1_w=1.375, emean1_b=-0.0625, emean2_w=0.875, emean2_b=0.5625,
        escale1_w=1.75, escale1_b=-0.5, escale2_w=0.625, escale2_b=-1.125,
        eps_q1=0.75, eps_q2=-1.25, eps_z=0.5625, eps_x=-0.8125,
    ),
    "B": dict(
        x1=4.0, x2=1.0,
        f_w_ih=0.5, f_b_ih=-0.0625, f_w_hh=-0.25, f_b_hh=0.125,
        b_w_ih=-1.5, b_b_ih=0.5, b_w_hh=0.875, b_b_hh=0.0,
        comb_w=-1.125, comb_b=0.375, mu_w=-0.875, mu_b=-0.25, sig_w=0.375, sig_b=-0.5, z0=-1.0,
        gate1_w=1.25, gate1_b=-0.375, gate2_w=2.0, gate2_b=-0.6875,
        prop1_w=0.5, prop1_b=-0.25, prop2_w=-1.75, prop2_b=-0.8125,
        lin_w=1.375, lin_b=-0.1875, tscale_w=-1.5, tscale_b=0.625,
        emean1_w=0.625, emean1_b=0.25, emean2_w=1.5, emean2_b=-0.125,
        escale1_w=-2.0, escale1_b=0.375, escale2_w=1.25, escale2_b=0.0625,
        eps_q1=-0.5, eps_q2=1.125, eps_z=-1.4375, eps_x=0.6875,
    ),
}


def relu(v):
    return v if v > 0.0 else 0.0


def softplus(v):
    return math.log1p(math.exp(v))  # arguments here are small; no overflow guard needed


def sigmoid(v):
    return 1.0 / (1.0 + math.exp(-v))


def work(p):
    o = {}
    # Sec. 3.1.3, last paragraph: observations are divided by twice the mean of the first window
    s = 2.0 * (p["x1"] + p["x2"]) / 2.0
    u1, u2 = p["x1"] / s, p["x2"] / s
    # guide: h_left runs over x_1, x_2; h_right over x_2, x_1 (ReLU RNNs, zero initial state)
    hl1 = relu(p["f_w_ih"] * u1 + p["f_b_ih"] + p["f_b_hh"])
    hl2 = relu(p["f_w_ih"] * u2 + p["f_b_ih"] + p["f_w_hh"] * hl1 + p["f_b_hh"])
    hr2 = relu(p["b_w_ih"] * u2 + p["b_b_ih"] + p["b_b_hh"])
    hr1 = relu(p["b_w_ih"] * u1 + p["b_b_ih"] + p["b_w_hh"] * hr2 + p["b_b_hh"])
    # guide, step 1: h_out = (tanh(W z_0 + b) + h_left + h_right) / 3; mu = K(h_out); sigma = softplus(L(mu))
    ho1 = (math.tanh(p["comb_w"] * p["z0"] + p["comb_b"]) + hl1 + hr1) / 3.0
    mu1 = p["mu_w"] * ho1 + p["mu_b"]
    sg1 = softplus(p["sig_w"] * mu1 + p["sig_b"])
    z1 = mu1 + sg1 * p["eps_q1"]
    # guide, step 2
    ho2 = (math.tanh(p["comb_w"] * z1 + p["comb_b"]) + hl2 + hr2) / 3.0
    mu2 = p["mu_w"] * ho2 + p["mu_b"]
    sg2 = softplus(p["sig_w"] * mu2 + p["sig_b"])
    zT = mu2 + sg2 * p["eps_q2"]
    # gated transition: g = sigmoid(W2 relu(W1 z + b1) + b2); h likewise without the sigmoid;
    # G = (1 - g)(W_l z + b_l) + g h;  H = softplus(W_s relu(G) + b_s)
    gate_hidden = p["gate1_w"] * zT + p["gate1_b"]
    g = sigmoid(p["gate2_w"] * relu(gate_hidden) + p["gate2_b"])
    prop_hidden = p["prop1_w"] * zT + p["prop1_b"]
    h = p["prop2_w"] * relu(prop_hidden) + p["prop2_b"]
    lin = p["lin_w"] * zT + p["lin_b"]
    G = (1.0 - g) * lin + g * h
    Hs = softplus(p["tscale_w"] * relu(G) + p["tscale_b"])
    zn = G + Hs * p["eps_z"]
    # emission: I = two affine layers (identity in between), J = softplus(W relu(W I + b) + b)
    I = p["emean2_w"] * (p["emean1_w"] * zn + p["emean1_b"]) + p["emean2_b"]
    I_relu = p["emean2_w"] * relu(p["emean1_w"] * zn + p["emean1_b"]) + p["emean2_b"]
    J = softplus(p["escale2_w"] * relu(p["escale1_w"] * I + p["escale1_b"]) + p["escale2_b"])
    x = s * (I + J * p["eps_x"])
    o.update(s=s, hl1=hl1, hl2=hl2, hr1=hr1, hr2=hr2, z_T=zT, gate_hidden=gate_hidden, g=g, h=h, lin=lin, G=G, H=Hs,
             z_next=zn, I=I, I_relu_variant=I_relu, J=J, x=x)
    return o


def main():
    lines = [
        "# The predictor of Sec. 3.1.3 with all widths 1 and a window of 2, worked as scalar arithmetic",
        "# by tests/golden/make_scalar_chain.py (math only; imports nothing of the repository).",
        "# in.<case>.<name>: inputs (exact in fp32).  out.<case>.<name>: what the equations give:",
        "#   s (normaliser, end of Sec. 3.1.3); hl*, hr* (RNN encodings of the guide); z_T (last guide step);",
        "#   gate_hidden, g, h, lin, G, H (gated transition display); z_next; I, J (emission display); x (seconds).",
    ]
    for name, p in CASES.items():
        for k, v in p.items():
            lines.append(f"in.{name}.{k} = {v!r}")
        for k, v in work(p).items():
            lines.append(f"out.{name}.{k} = {v!r}")
    out = Path(__file__).resolve().parent / "scalar_chain.txt"
    out.write_text("\n".join(lines) + "\n")
    print(f"wrote {out}")


if __name__ == "__main__":
    main()
