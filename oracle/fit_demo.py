"""Fit a preset on the first part of its synthetic trace, then replay the held-out part through the
CPU oracle and print gradients per second for: the predictor's cutoffs, waiting for everyone, the
best single fixed cutoff in hindsight, and the per-step hindsight optimum (Sec. 4.1's comparison,
on synthetic traces that stand in for the paper's cluster recordings).

    python -m oracle.fit_demo --preset replay --train 600 --steps 1500

CPU only; test infrastructure like the rest of this package.
"""
from __future__ import annotations

import argparse
import time

import numpy as np

import cluster_synth as synth

from . import binding, elbo


def replay(cfg, blob, trace, first, samples, stride=1):
    """Cutoffs the oracle predictor chooses for steps first+1.. of `trace`, deciding every `stride` steps."""
    m = binding.OracleModel(cfg, blob)
    steps, chosen = [], []
    for t in range(trace.shape[0] - 1):
        m.filter_step(trace[t])
        if t >= first and t >= cfg.lag - 1 and (t - first) % stride == 0:
            eq, ez, ex = synth.make_noise(cfg, samples=samples, draw=t)
            c, _ = m.predict_cutoff(eq, ez, ex)
            steps.append(t + 1)
            chosen.append(c)
    m.close()
    return np.array(steps), np.array(chosen, dtype=np.int32)


def report(trace, steps, chosen):
    rows = trace[steps]
    got, full, hindsight = binding.trace_throughput(rows, chosen)
    srt = np.sort(rows.astype(np.float64), axis=1)
    N = rows.shape[1]
    fixed = max(k * len(steps) / srt[:, k - 1].sum() for k in range(1, N + 1))
    return dict(chosen=got, full_sync=full, best_fixed=float(fixed), hindsight=hindsight,
                c_min=int(chosen.min()), c_median=float(np.median(chosen)), c_max=int(chosen.max()))


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--preset", default="replay", choices=sorted(synth.CONFIGS))
    ap.add_argument("--train", type=int, default=600, help="trace steps used for fitting")
    ap.add_argument("--steps", type=int, default=1500, help="optimiser steps")
    ap.add_argument("--lr", type=float, default=2e-3)
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--samples", type=int, default=512)
    ap.add_argument("--stride", type=int, default=4, help="decide every this many held-out steps")
    a = ap.parse_args()
    cfg = synth.CONFIGS[a.preset]
    trace = synth.make_trace(cfg)
    blob = synth.make_blob(cfg)
    t0 = time.time()
    fitted, hist = elbo.fit(cfg, blob, trace[:a.train], steps=a.steps, lr=a.lr, batch=a.batch, seed=3,
                            log=max(1, a.steps // 10))
    print(f"fit: {time.time() - t0:.0f} s, ELBO per window {np.mean(hist[:20]):.4g} -> {np.mean(hist[-20:]):.4g}")
    for name, b in (("random weights", blob), ("fitted weights", fitted)):
        steps, chosen = replay(cfg, b, trace, a.train, a.samples, a.stride)
        print(name, report(trace, steps, chosen), flush=True)


if __name__ == "__main__":
    main()
