"""Seeded synthetic inputs: cluster presets, weight blobs, run-time traces, noise.

This module only *draws numbers and lays them out*; it holds none of the
method's arithmetic and is the one piece of code that both the GPU library's
tests and the CPU oracle's tests feed from.

The presets stand in for the recorded cluster traces of the paper's
experiments (Sec. 4.1: a 158-worker Xeon cluster and a 2175-worker KNL
machine), which are not public.  They reproduce the regimes the paper
describes (Sec. 2.1): iid jitter, independent stragglers, and persistent
slowdowns shared by all workers of a node.

Weight blob format (little endian):
    int32[8]  : magic 'DKFW', version, N, L, Z, H, R, 0
    float32[] : the tensors of `blob_layout`, in that order, each row-major;
                a matrix is stored [out][in] so that a layer is  W x + b
                (the paper's MLP_n / RNN notation, Sec. 3.1.3).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Tuple

import numpy as np

BLOB_MAGIC = 0x57464B44  # 'DKFW'
BLOB_VERSION = 1
BLOB_HEADER_INTS = 8
SEED_BASE = 180304209 * 10


@dataclass(frozen=True)
class ClusterConfig:
    """One predictor configuration (N workers, lag L, latent Z, hidden H, RNN R)."""

    name: str
    index: int  # 1-based preset number, enters the seed
    n_workers: int
    lag: int
    z_dim: int
    hidden: int
    rnn_dim: int
    samples: int
    mlp_dtype: str  # "f32" or "bf16"
    trace_len: int
    trace_kind: str

    @property
    def seed(self) -> int:
        return SEED_BASE + self.index

    def with_samples(self, s: int) -> "ClusterConfig":
        return replace(self, samples=int(s))


CONFIGS: Dict[str, ClusterConfig] = {
    c.name: c
    for c in [
        ClusterConfig("tiny", 1, 16, 5, 8, 32, 32, 256, "f32", 200, "iid_stragglers_tiny"),
        ClusterConfig("medium", 2, 128, 10, 16, 128, 128, 4096, "f32", 1000, "iid_stragglers_medium"),
        ClusterConfig("contended", 3, 512, 10, 32, 256, 256, 16384, "f32", 2000, "grouped_markov"),
        ClusterConfig("large_bf16", 4, 2048, 20, 64, 512, 512, 8192, "bf16", 1000, "racks_pareto"),
        ClusterConfig("replay", 5, 512, 10, 32, 256, 256, 4096, "f32", 1010, "grouped_markov"),
    ]
}


def blob_layout(cfg: ClusterConfig) -> List[Tuple[str, Tuple[int, ...]]]:
    """Names and shapes of the blob tensors, in storage order."""
    N, Z, H, R = cfg.n_workers, cfg.z_dim, cfg.hidden, cfg.rnn_dim
    return [
        # inference network: forward ("left") and backward ("right") ReLU RNNs
        ("rnn_f_w_ih", (R, N)), ("rnn_f_b_ih", (R,)), ("rnn_f_w_hh", (R, R)), ("rnn_f_b_hh", (R,)),
        ("rnn_b_w_ih", (R, N)), ("rnn_b_b_ih", (R,)), ("rnn_b_w_hh", (R, R)), ("rnn_b_b_hh", (R,)),
        # inference network: combiner, mean and scale heads, initial latent
        ("comb_w", (R, Z)), ("comb_b", (R,)),
        ("mu_w", (Z, R)), ("mu_b", (Z,)),
        ("sig_w", (Z, Z)), ("sig_b", (Z,)),
        ("z0", (Z,)),
        # gated transition
        ("gate1_w", (H, Z)), ("gate1_b", (H,)), ("gate2_w", (Z, H)), ("gate2_b", (Z,)),
        ("prop1_w", (H, Z)), ("prop1_b", (H,)), ("prop2_w", (Z, H)), ("prop2_b", (Z,)),
        ("lin_w", (Z, Z)), ("lin_b", (Z,)),
        ("tscale_w", (Z, Z)), ("tscale_b", (Z,)),
        # emission: mean I (two layers) and scale J (two layers, fed by the mean)
        ("emean1_w", (H, Z)), ("emean1_b", (H,)), ("emean2_w", (N, H)), ("emean2_b", (N,)),
        ("escale1_w", (H, N)), ("escale1_b", (H,)), ("escale2_w", (N, H)), ("escale2_b", (N,)),
    ]


def blob_num_floats(cfg: ClusterConfig) -> int:
    return int(sum(int(np.prod(s)) for _, s in blob_layout(cfg)))


def pack_blob(cfg: ClusterConfig, tensors: Dict[str, np.ndarray]) -> np.ndarray:
    """Serialise named tensors into one uint8 blob (header + fp32 payload)."""
    head = np.array(
        [BLOB_MAGIC, BLOB_VERSION, cfg.n_workers, cfg.lag, cfg.z_dim, cfg.hidden, cfg.rnn_dim, 0],
        dtype="<i4",
    )
    parts = []
    for name, shape in blob_layout(cfg):
        t = np.asarray(tensors[name], dtype="<f4")
        if t.shape != tuple(shape):
            raise ValueError(f"{name}: shape {t.shape}, expected {shape}")
        parts.append(np.ascontiguousarray(t).reshape(-1))
    body = np.concatenate(parts)
    return np.concatenate([head.view(np.uint8), body.view(np.uint8)])


def unpack_blob(cfg: ClusterConfig, blob: np.ndarray) -> Dict[str, np.ndarray]:
    """Inverse of `pack_blob` (copies)."""
    raw = np.ascontiguousarray(blob).view(np.uint8)
    body = raw[BLOB_HEADER_INTS * 4:].view("<f4")
    out, off = {}, 0
    for name, shape in blob_layout(cfg):
        n = int(np.prod(shape))
        out[name] = body[off:off + n].reshape(shape).copy()
        off += n
    if off != body.size:
        raise ValueError("blob size does not match the configuration")
    return out


def _streams(cfg: ClusterConfig):
    """Independent generators for weights, trace and noise of one preset."""
    ss = np.random.SeedSequence(cfg.seed).spawn(3)
    return [np.random.Generator(np.random.PCG64(s)) for s in ss]


def make_weights(cfg: ClusterConfig, std: float = 0.1, calibrated: bool = False) -> Dict[str, np.ndarray]:
    """Every tensor, biases and z0 included, iid N(0, std^2) in fp32.

    `calibrated` adds fixed offsets to the output biases of the emission networks so that the
    predicted run-times sit near 0.5 in units of the normaliser (where real run-times sit, the
    normaliser being twice their mean) with a spread of 0.05 for the small presets (wide hidden
    layers add to it), instead of scattering around zero."""
    g = _streams(cfg)[0]
    w = {
        name: (std * g.standard_normal(shape)).astype(np.float32)
        for name, shape in blob_layout(cfg)
    }
    if calibrated:
        w["emean2_b"] = (w["emean2_b"] + np.float32(0.5)).astype(np.float32)
        w["escale2_b"] = (w["escale2_b"] + np.float32(CALIBRATED_SCALE_BIAS)).astype(np.float32)
    return w


# softplus(-2.97) = 0.050
CALIBRATED_SCALE_BIAS = -2.97


def make_blob(cfg: ClusterConfig, std: float = 0.1, calibrated: bool = False) -> np.ndarray:
    return pack_blob(cfg, make_weights(cfg, std, calibrated))


def _markov_groups(g, T: int, groups: int, stay: float, slow: float) -> np.ndarray:
    """[T][groups] multipliers from 2-state chains started in the stationary law."""
    state = g.random(groups) < 0.5
    out = np.empty((T, groups), dtype=np.float64)
    for t in range(T):
        out[t] = np.where(state, slow, 1.0)
        flip = g.random(groups) >= stay
        state = np.logical_xor(state, flip)
    return out


def make_trace(cfg: ClusterConfig, length: int | None = None) -> np.ndarray:
    """Synthetic run-times in seconds, float32 [T][N], strictly positive."""
    g = _streams(cfg)[1]
    T = int(length if length is not None else cfg.trace_len)
    N = cfg.n_workers
    kind = cfg.trace_kind
    if kind == "iid_stragglers_tiny":
        x = 1.0 * np.exp(0.1 * g.standard_normal((T, N)))
        hit = g.random((T, N)) < 0.1
        x = np.where(hit, x * g.uniform(2.0, 4.0, (T, N)), x)
    elif kind == "iid_stragglers_medium":
        x = 0.5 * np.exp(0.15 * g.standard_normal((T, N)))
        hit = g.random((T, N)) < 0.05
        x = np.where(hit, x * g.uniform(1.5, 5.0, (T, N)), x)
    elif kind == "grouped_markov":
        groups = 8
        per = N // groups
        m = _markov_groups(g, T, groups, 0.95, 2.0)
        x = 1.0 * np.exp(0.1 * g.standard_normal((T, N))) * np.repeat(m, per, axis=1)
    elif kind == "racks_pareto":
        racks = 32
        per = N // racks
        m = _markov_groups(g, T, racks, 0.95, 2.0)
        x = 2.0 * np.exp(0.2 * g.standard_normal((T, N))) * np.repeat(m, per, axis=1)
        hit = g.random((T, N)) < 0.01
        tail = (1.0 - g.random((T, N))) ** (-1.0 / 1.5)
        x = np.where(hit, x * tail, x)
    else:
        raise ValueError(kind)
    return x.astype(np.float32)


def make_noise(cfg: ClusterConfig, samples: int | None = None, draw: int = 0):
    """Standard-normal fp32 tensors (eps_q [L][S][Z], eps_z [S][Z], eps_x [S][N]).

    `draw` selects an independent set (one per decision step)."""
    S = int(samples if samples is not None else cfg.samples)
    ss = np.random.SeedSequence(cfg.seed).spawn(3)[2]
    g = np.random.Generator(np.random.PCG64(ss.spawn(draw + 1)[draw]))
    eps_q = g.standard_normal((cfg.lag, S, cfg.z_dim), dtype=np.float32)
    eps_z = g.standard_normal((S, cfg.z_dim), dtype=np.float32)
    eps_x = g.standard_normal((S, cfg.n_workers), dtype=np.float32)
    return eps_q, eps_z, eps_x


def make_runtime_matrix(kind: str, S: int, N: int, seed: int) -> np.ndarray:
    """Sample matrices [S][N] (fp32) for exercising the order-statistics stage alone."""
    g = np.random.Generator(np.random.PCG64(seed))
    if kind == "uniform":
        x = g.random((S, N))
    elif kind == "exponential":
        x = g.standard_exponential((S, N))
    elif kind == "normal":
        x = g.standard_normal((S, N))
    elif kind == "lognormal_stragglers":
        x = np.exp(0.15 * g.standard_normal((S, N)))
        hit = g.random((S, N)) < 0.05
        x = np.where(hit, x * g.uniform(1.5, 5.0, (S, N)), x)
    elif kind == "ties":
        x = g.integers(0, 4, (S, N)).astype(np.float64) * 0.25 + 0.25
    elif kind == "signed_zeros":
        x = g.standard_normal((S, N))
        x[g.random((S, N)) < 0.2] = 0.0
        x[g.random((S, N)) < 0.2] = -0.0
    else:
        raise ValueError(kind)
    return x.astype(np.float32)
