"""Pins for the two sub-networks of Sec. 3.1.3 whose weights act at ordinary (non-degenerate)
values: the gate g = MLP_2(z, ReLU, Sigmoid) of the transition and the combiner term W z inside
the tanh of the guide -- CPU only.

None of these compares the oracle with a re-typing of its loops:
  * two hand-worked cases with small integer matrices (non-square, so a transposed operand
    fails) whose expected values are literal numbers derived in the comments from
    sigmoid(log 3) = 3/4, tanh(log 2) = 3/5, tanh(log 3) = 4/5, softplus(log(e^a - 1)) = a;
  * the all-widths-one chain worked as scalar arithmetic by tests/golden/make_scalar_chain.py
    (math only), read from tests/golden/scalar_chain.txt;
  * the limit of a steep gate, where g becomes a step function of |z + b| and G switches between
    the linear and the proposed mean.
The biases built from logarithms are rounded to fp32 in the weight blob, hence the 1e-5 absolute
tolerance of the hand-worked cases (a planted mistake moves them by 0.1 or more).
Planted mistakes each of them must catch are exercised at the end (on the CPU, in a mutated copy
of the oracle's source).
"""
import math
import re
import subprocess
from pathlib import Path

import numpy as np
import pytest

import oracle
import cluster_synth as synth

ROOT = Path(__file__).resolve().parents[1]
LOG2, LOG3 = math.log(2.0), math.log(3.0)


def inv_softplus(a):
    return math.log(math.expm1(a))


def cfg_of(N, L, Z, H, R, S=1):
    return synth.ClusterConfig("pin", 7, N, L, Z, H, R, S, "f32", 10, "iid_stragglers_tiny")


def zero_weights(cfg):
    return {name: np.zeros(shape, dtype=np.float32) for name, shape in synth.blob_layout(cfg)}


def model(cfg, w, window, act=0, mod=oracle):
    m = mod.OracleModel(cfg, synth.pack_blob(cfg, w), emit_mean_act=act)
    for row in window:
        m.filter_step(np.asarray(row, dtype=np.float64))
    return m


# ---- hand-worked case 1: gated transition and emission, Z = 2, H = 3, N = 2 ---------------------

def transition_case():
    cfg = cfg_of(N=2, L=1, Z=2, H=3, R=2)
    w = zero_weights(cfg)
    # guide switched to a constant: mu_q = b_mu, no noise  =>  z_T = (1, -2)
    w["mu_b"][:] = [1, -2]
    # gate: W1 z + b1 = (1 + .5, -2 + 1, 1 - 2) = (1.5, -1, -1); ReLU -> (1.5, 0, 0)
    w["gate1_w"][:] = [[1, 0], [0, 1], [1, 1]]
    w["gate1_b"][:] = [0.5, 1, 0]
    # W2 (1.5, 0, 0) = (3, -1.5); b2 chosen so that the sigmoid's argument is (log 3, -log 3): g = (3/4, 1/4)
    w["gate2_w"][:] = [[2, 5, -3], [-1, 4, 7]]
    w["gate2_b"][:] = [LOG3 - 3, 1.5 - LOG3]
    # proposed mean: W1 z + b1 = (-1 - 4, 3 - 2, 2 + 1) = (-5, 1, 3); ReLU -> (0, 1, 3);
    # h = (0 + 1 + 6 + .5, 0 - 2 + 3 - 1) = (7.5, 0)
    w["prop1_w"][:] = [[-1, 2], [3, 1], [0, -1]]
    w["prop1_b"][:] = [0, 0, 1]
    w["prop2_w"][:] = [[4, 1, 2], [9, -2, 1]]
    w["prop2_b"][:] = [0.5, -1]
    # linear part: (2 - 2, -1 - 6 + 1) = (0, -6)
    w["lin_w"][:] = [[2, 1], [-1, 3]]
    w["lin_b"][:] = [0, 1]
    # G = (1/4 * 0 + 3/4 * 7.5, 3/4 * -6 + 1/4 * 0) = (5.625, -4.5); ReLU(G) = (5.625, 0);
    # W_s ReLU(G) = (2.8125, -1.40625); b_s chosen so that H = softplus(.) = (2, 1)
    w["tscale_w"][:] = [[0.5, 3], [-0.25, 2]]
    w["tscale_b"][:] = [inv_softplus(2.0) - 2.8125, inv_softplus(1.0) + 1.40625]
    # z_{T+1} = G + H eps_z = (5.625 + 2 * .5, -4.5 + 1 * -2) = (6.625, -6.5)
    # emission mean: hidden = (6.625, -6.5, 2 * .125 - .25) = (6.625, -6.5, 0) (identity in between);
    # I = (13.25 - 6.5 + .25, 6.5 - .5) = (7, 6);  ReLU variant: hidden (6.625, 0, 0), I = (13.5, -0.5)
    w["emean1_w"][:] = [[1, 0], [0, 1], [2, 2]]
    w["emean1_b"][:] = [0, 0, -0.25]
    w["emean2_w"][:] = [[2, 1, 5], [0, -1, 3]]
    w["emean2_b"][:] = [0.25, -0.5]
    # scale: W1 I + b1 = (7 - 6, -1, 6.5 - 6) = (1, -1, .5); ReLU -> (1, 0, .5); W2 . = (3 + 1, -2 + 2) = (4, 0);
    # b2 chosen so that J = (3, 1/2)
    w["escale1_w"][:] = [[1, -1], [-1, 1], [0.5, 0.5]]
    w["escale1_b"][:] = [0, 0, -6]
    w["escale2_w"][:] = [[3, 9, 2], [-2, 9, 4]]
    w["escale2_b"][:] = [inv_softplus(3.0) - 4, inv_softplus(0.5)]
    window = [[3.0, 5.0]]  # s = 2 * mean = 8
    eq = np.zeros((1, 1, 2), np.float32)
    ez = np.array([[0.5, -2.0]], np.float32)
    ex = np.array([[-1.0, 2.0]], np.float32)
    return cfg, w, window, (eq, ez, ex)


TRANSITION_EXPECT = dict(z_T=[1, -2], gate_hidden=[1.5, -1, -1], gate_pre=[LOG3, -LOG3], gate=[0.75, 0.25],
                         prop=[7.5, 0], lin=[0, -6], G=[5.625, -4.5], Hs=[2, 1], z_next=[6.625, -6.5],
                         emit_mean=[7, 6], emit_sd=[3, 0.5], x=[8 * (7 - 3), 8 * (6 + 1)])


def run_transition_case(mod=oracle, act=0):
    cfg, w, window, (eq, ez, ex) = transition_case()
    m = model(cfg, w, window, act=act, mod=mod)
    x, st = m.sample_runtimes(eq, ez, ex, stages=True)
    got = dict(st, x=x, **m.transition_terms(eq, ez, ex))
    return m, got


def test_hand_worked_transition_and_emission():
    m, got = run_transition_case()
    assert m.scale == 8.0
    for k, v in TRANSITION_EXPECT.items():
        assert np.allclose(got[k][0], v, rtol=2e-6, atol=1e-5), (k, got[k][0], v)


def test_hand_worked_emission_relu_variant():
    _, got = run_transition_case(act=1)
    assert np.allclose(got["emit_mean"][0], [13.5, -0.5], rtol=2e-6, atol=1e-5)


# ---- hand-worked case 2: the combiner of the guide, Z = 2, R = 3 ---------------------------------

def combiner_case():
    cfg = cfg_of(N=2, L=1, Z=2, H=1, R=3)
    w = zero_weights(cfg)
    # x / s = (3, 5) / 8; forward: W x / s = (3, 5, -2), + b_ih + b_hh = (4.5, 4, -1.25); ReLU -> (4.5, 4, 0)
    w["rnn_f_w_ih"][:] = [[8, 0], [0, 8], [8, -8]]
    w["rnn_f_b_ih"][:] = [1, -1, 0.5]
    w["rnn_f_b_hh"][:] = [0.5, 0, 0.25]
    # backward: (5, -3, 0) + (0.25, 3.5, -2) = (5.25, .5, -2); ReLU -> (5.25, .5, 0)
    w["rnn_b_w_ih"][:] = [[0, 8], [-8, 0], [0, 0]]
    w["rnn_b_b_ih"][:] = [0.25, 3.5, -2]
    # combiner: W z0 = (1 - 2, 3 - 1, 2 - 2) = (-1, 2, 0); b chosen so that the tanh's argument is
    # (log 2, -log 3, 0): tanh = (3/5, -4/5, 0)
    w["z0"][:] = [1, -1]
    w["comb_w"][:] = [[1, 2], [3, 1], [2, 2]]
    w["comb_b"][:] = [LOG2 + 1, -LOG3 - 2, 0]
    # h_out = ((.6 + 4.5 + 5.25) / 3, (-.8 + 4 + .5) / 3, 0) = (3.45, 37/30, 0)
    # mu = (2 * 3.45 + 3 * 37/30 + .125, -3.45 + 6 * 37/30 - .375) = (10.725, 3.575)
    w["mu_w"][:] = [[2, 3, 7], [-1, 6, 1]]
    w["mu_b"][:] = [0.125, -0.375]
    # sigma = softplus(W mu + b) with W mu = (10.725 - 7.15, 7.15) = (3.575, 7.15), b chosen so that sigma = (2, 1/2)
    w["sig_w"][:] = [[1, -2], [0, 2]]
    w["sig_b"][:] = [inv_softplus(2.0) - 3.575, inv_softplus(0.5) - 7.15]
    # z_T = mu + sigma eps = (10.725 + 2 * 1.5, 3.575 + .5 * -3) = (13.725, 2.075)
    eq = np.array([[[1.5, -3.0]]], np.float32)
    return cfg, w, [[3.0, 5.0]], (eq, np.zeros((1, 2), np.float32), np.zeros((1, 2), np.float32))


def run_combiner_case(mod=oracle):
    cfg, w, window, (eq, ez, ex) = combiner_case()
    m = model(cfg, w, window, mod=mod)
    hl, hr = m.encode_window()
    _, st = m.sample_runtimes(eq, ez, ex, stages=True)
    return hl, hr, st["z_T"]


def test_hand_worked_combiner():
    hl, hr, zT = run_combiner_case()
    assert np.allclose(hl[0], [4.5, 4, 0], atol=1e-12) and np.allclose(hr[0], [5.25, 0.5, 0], atol=1e-12)
    assert np.allclose(zT[0], [13.725, 2.075], rtol=2e-6, atol=1e-5)


# ---- the all-widths-one chain, worked by a math-only script ----------------------------------------

def read_scalar_cases(golden_dir):
    cases = {}
    for line in (golden_dir / "scalar_chain.txt").read_text().splitlines():
        mt = re.match(r"(in|out)\.(\w+?)\.(\w+) = (\S+)$", line)
        if mt:
            cases.setdefault(mt.group(2), {"in": {}, "out": {}})[mt.group(1)][mt.group(3)] = float(mt.group(4))
    return cases


SCALAR_NAMES = {"f_w_ih": "rnn_f_w_ih", "f_b_ih": "rnn_f_b_ih", "f_w_hh": "rnn_f_w_hh", "f_b_hh": "rnn_f_b_hh",
                "b_w_ih": "rnn_b_w_ih", "b_b_ih": "rnn_b_b_ih", "b_w_hh": "rnn_b_w_hh", "b_b_hh": "rnn_b_b_hh"}


def run_scalar_case(inp, act=0, mod=oracle):
    cfg = cfg_of(N=1, L=2, Z=1, H=1, R=1)
    w = zero_weights(cfg)
    for k, v in inp.items():
        name = SCALAR_NAMES.get(k, k)
        if name in w:
            assert np.float32(v) == v  # exact in fp32
            w[name][...] = v
    m = model(cfg, w, [[inp["x1"]], [inp["x2"]]], act=act, mod=mod)
    eq = np.array([[[inp["eps_q1"]]], [[inp["eps_q2"]]]], np.float32)
    ez = np.array([[inp["eps_z"]]], np.float32)
    ex = np.array([[inp["eps_x"]]], np.float32)
    hl, hr = m.encode_window()
    x, st = m.sample_runtimes(eq, ez, ex, stages=True)
    t = m.transition_terms(eq, ez, ex)
    return dict(s=m.scale, hl1=hl[0, 0], hl2=hl[1, 0], hr1=hr[0, 0], hr2=hr[1, 0], z_T=st["z_T"][0, 0],
                gate_hidden=t["gate_hidden"][0, 0], g=t["gate"][0, 0], h=t["prop"][0, 0], lin=t["lin"][0, 0],
                G=t["G"][0, 0], H=t["Hs"][0, 0], z_next=st["z_next"][0, 0], I=st["emit_mean"][0, 0],
                J=st["emit_sd"][0, 0], x=x[0, 0])


@pytest.mark.parametrize("case", ["A", "B"])
def test_scalar_chain_matches_the_worked_values(golden_dir, case):
    c = read_scalar_cases(golden_dir)[case]
    got = run_scalar_case(c["in"])
    for k, v in got.items():
        assert v == pytest.approx(c["out"][k], rel=1e-12, abs=1e-14), k
    got_relu = run_scalar_case(c["in"], act=1)
    assert got_relu["I"] == pytest.approx(c["out"]["I_relu_variant"], rel=1e-12, abs=1e-14)


def test_scalar_cases_switch_their_relus_both_ways(golden_dir):
    c = read_scalar_cases(golden_dir)
    assert c["A"]["out"]["gate_hidden"] > 0 > c["B"]["out"]["gate_hidden"]
    assert c["A"]["out"]["G"] > 0 > c["B"]["out"]["G"]
    assert c["A"]["out"]["hr1"] > 0 == c["B"]["out"]["hr1"]
    assert c["B"]["out"]["I"] != c["B"]["out"]["I_relu_variant"]


# ---- limit of a steep gate ----------------------------------------------------------------------------

def steep_gate_weights(cfg, kappa, theta):
    Z = cfg.z_dim
    assert cfg.hidden == 2 * Z
    w = synth.make_weights(cfg, std=0.5)
    # hidden units (ReLU(z + b), ReLU(-z - b)), output kappa (|z + b| - theta): g -> 1 where |z + b| > theta
    b = w["gate1_b"][:Z].copy()
    w["gate1_w"][:] = np.vstack([np.eye(Z), -np.eye(Z)])
    w["gate1_b"][:] = np.concatenate([b, -b])
    w["gate2_w"][:] = kappa * np.hstack([np.eye(Z), np.eye(Z)])
    w["gate2_b"][:] = -kappa * theta
    return w, b.astype(np.float64)


def test_steep_gate_switches_between_linear_and_proposed_mean():
    cfg = cfg_of(N=5, L=3, Z=4, H=8, R=6, S=400)
    theta = 0.4
    w, b = steep_gate_weights(cfg, kappa=4096.0, theta=theta)
    m = model(cfg, w, synth.make_trace(cfg)[:cfg.lag])
    eq, ez, ex = synth.make_noise(cfg)
    _, st = m.sample_runtimes(eq, ez, ex, stages=True)
    t = m.transition_terms(eq, ez, ex)
    d = {k: v.astype(np.float64) for k, v in w.items()}
    zT = st["z_T"]
    margin = np.abs(zT + b) - theta
    sure = np.abs(margin) > 0.02  # away from the switching point the sigmoid is 0 or 1 to 1e-35
    assert sure.mean() > 0.9 and (margin[sure] > 0).any() and (margin[sure] < 0).any()
    assert np.array_equal(t["gate"][sure] > 0.5, margin[sure] > 0)
    assert np.all(np.minimum(t["gate"][sure], 1 - t["gate"][sure]) < 1e-30)
    # G is the proposed mean where the gate is open and the linear mean where it is shut: both
    # taken from the oracle's own taps, which the hand-worked case pins
    assert np.allclose(t["G"][sure], np.where(margin > 0, t["prop"], t["lin"])[sure], rtol=1e-12, atol=1e-14)
    lin = zT @ d["lin_w"].T + d["lin_b"]
    assert np.allclose(t["lin"], lin, rtol=1e-12, atol=1e-13)
    rows = sure.all(axis=1)
    assert np.allclose(st["z_next"][rows], (t["G"] + t["Hs"] * ez)[rows], rtol=1e-12, atol=1e-13)


# ---- planted mistakes: each must be caught by a test above that is not a transcription -----------

MUTATIONS = {
    "gate ReLU dropped":
        ("    for (int i = 0; i < H; ++i) w->hid[i] = relu(w->hid[i]);\n    mlp_layer(m, m->gate2_w,",
         "    mlp_layer(m, m->gate2_w,"),
    "sigmoid replaced by (1 + tanh)/2":
        ("for (int i = 0; i < Z; ++i) w->g[i] = sigmoid(w->g[i]);",
         "for (int i = 0; i < Z; ++i) w->g[i] = 0.5 * (1.0 + tanh(w->g[i]));"),
    "gate fed the proposed mean's first layer":
        ("mlp_layer(m, m->gate1_w, m->gate1_b, w->z, Z, H, w->hid, w->xq);",
         "mlp_layer(m, m->prop1_w, m->gate1_b, w->z, Z, H, w->hid, w->xq);"),
    "gate and (1 - gate) swapped":
        ("(1.0 - w->g[i]) * w->lin[i] + w->g[i] * w->h[i]", "w->g[i] * w->lin[i] + (1.0 - w->g[i]) * w->h[i]"),
    "combiner ignores the previous latent":
        ("mlp_layer(m, m->comb_w, m->comb_b, w->z, Z, R, w->r1, w->xq);",
         "mlp_layer(m, m->comb_w, m->comb_b, m->z0, Z, R, w->r1, w->xq);"),
    "combiner divided by two":
        ("H_RIGHT(t, r)) / 3.0;", "H_RIGHT(t, r)) / 2.0;"),
    "transition scale fed G instead of ReLU(G)":
        ("for (int i = 0; i < Z; ++i) w->mu[i] = relu(w->G[i]);", "for (int i = 0; i < Z; ++i) w->mu[i] = w->G[i];"),
    "emission scale fed z instead of the mean":
        ("mlp_layer(m, m->escale1_w, m->escale1_b, w->mean, N, H, w->hid, w->xq);",
         "mlp_layer(m, m->escale1_w, m->escale1_b, w->zn, N, H, w->hid, w->xq);"),
}


class _Mutant:
    """The oracle's binding over a mutated copy of its C source (CPU only)."""

    def __init__(self, tmp_path, old, new, defines=()):
        import ctypes as C

        from oracle import binding

        src = (ROOT / "oracle" / "cutoff_oracle.c").read_text()
        if old is not None:
            assert src.count(old) == 1, old
            src = src.replace(old, new)
        c_file = tmp_path / "mutant.c"
        c_file.write_text(src)
        so = tmp_path / "libmutant.so"
        subprocess.run(["gcc", "-std=c99", "-O1", "-fopenmp", "-fPIC", "-shared", *defines, "-o", str(so), str(c_file),
                        "-lm"], check=True)
        self._binding, self._saved, self._C, self._so = binding, binding._lib, C, so

    def __enter__(self):
        b = self._binding
        b._lib = None
        saved_path = b._LIB
        b._LIB = self._so
        real_build = b.build
        b.build = lambda force=False: self._so
        try:
            b._load()
        finally:
            b._LIB, b.build = saved_path, real_build
        return b

    def __exit__(self, *exc):
        self._binding._lib = self._saved


@pytest.mark.parametrize("name", list(MUTATIONS))
def test_planted_mistake_is_caught(tmp_path, golden_dir, name):
    old, new = MUTATIONS[name]
    cases = read_scalar_cases(golden_dir)
    with _Mutant(tmp_path, old, new) as mod:
        failures = []
        _, got = run_transition_case(mod=mod)
        if not all(np.allclose(got[k][0], v, rtol=2e-6, atol=1e-5) for k, v in TRANSITION_EXPECT.items()):
            failures.append("hand-worked transition")
        if not np.allclose(run_combiner_case(mod=mod)[2][0], [13.725, 2.075], rtol=2e-6, atol=1e-5):
            failures.append("hand-worked combiner")
        for case in ("A", "B"):
            got = run_scalar_case(cases[case]["in"], mod=mod)
            if not all(v == pytest.approx(cases[case]["out"][k], rel=1e-12, abs=1e-14) for k, v in got.items()):
                failures.append(f"scalar chain {case}")
    assert failures, f"no pin noticed: {name}"


def test_literal_reading_of_the_encodings_skips_the_observation_of_its_own_step(tmp_path):
    """Sec. 3.1.3 prints h_left over x_{T-l:t-1} and h_right over x_{t+1:T}: the guide's step t would
    then not use x_t itself.  Built that way (-DORACLE_A8_LITERAL) a window of one observation has
    no influence on the prediction at all, and in a longer window the newest observation reaches
    z_T only through the earlier latents; with the reading taken (both encodings include x_t) the
    last step sees it directly."""
    eq1 = np.zeros((1, 8, 3), np.float32)
    cfg1 = cfg_of(N=4, L=1, Z=3, H=5, R=6, S=8)
    w1 = synth.make_weights(cfg1, std=0.5)
    x_a, x_b = np.array([1.0, 2.0, 3.0, 4.0]), np.array([4.0, 1.0, 2.0, 3.0])  # same mean: same normaliser
    noise1 = (eq1, *synth.make_noise(cfg1)[1:])

    def z_T(mod, cfg, w, window, noise):
        _, st = model(cfg, w, window, mod=mod).sample_runtimes(*noise, stages=True)
        return st["z_T"]

    assert not np.allclose(z_T(oracle, cfg1, w1, [x_a], noise1), z_T(oracle, cfg1, w1, [x_b], noise1))
    cfg3 = cfg_of(N=4, L=3, Z=3, H=5, R=6, S=8)
    w3 = synth.make_weights(cfg3, std=0.5)
    w3["comb_w"][:] = 0  # cut the chain: z_t no longer depends on z_{t-1}
    noise3 = synth.make_noise(cfg3)
    win_a, win_b = [x_b, x_a, x_a], [x_b, x_a, x_b]  # differ in the newest observation only
    assert not np.allclose(z_T(oracle, cfg3, w3, win_a, noise3), z_T(oracle, cfg3, w3, win_b, noise3))
    with _Mutant(tmp_path, None, None, defines=("-DORACLE_A8_LITERAL",)) as literal:
        one_a, one_b = z_T(literal, cfg1, w1, [x_a], noise1), z_T(literal, cfg1, w1, [x_b], noise1)
        three_a, three_b = z_T(literal, cfg3, w3, win_a, noise3), z_T(literal, cfg3, w3, win_b, noise3)
        three_c = z_T(literal, cfg3, w3, [x_b, x_b, x_a], noise3)  # the middle observation does reach z_T
    assert np.array_equal(one_a, one_b)
    assert np.array_equal(three_a, three_b) and not np.allclose(three_a, three_c)
