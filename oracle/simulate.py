"""Discrete-event simulation of the parameter-server loop of Alg. 1, driven by a run-time trace.

Test infrastructure (CPU, plain Python/numpy): it turns a sequence of cutoffs into simulated
wall-clock time, with the feedback the server really has — the run-times of the workers it waited
for, and only a lower bound for the ones it cut off (Sec. 4.2).

One iteration, as the server of Alg. 1 sees it:
  1. c <- policy.decide()                                  (predict_cutoff)
  2. every worker starts; worker w finishes trace[t][w] seconds later (an event in a time-ordered queue)
  3. the server takes finish events in time order until it holds c of them; each carries the
     worker's gradient and its measured run-time
  4. the participants are published as a bit array; the others are terminated, their gradients
     count as zero, and the update is theta <- theta - alpha * (1/c) * (sum over all workers of the
     masked gradients)   (Sec. 4.1, last paragraph: bit array + all-reduce form of the same update)
  5. the clock advances by the c-th smallest run-time plus a fixed per-iteration overhead
  6. policy.observe(run-times, censored mask, censoring time)

Equal finish times are taken in worker order (the order of equal keys in the cutoff rule's sort).
"""
from __future__ import annotations

import heapq
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from . import binding


class FullSync:
    """Wait for everybody."""

    def __init__(self, n):
        self.n = n

    def decide(self):
        return self.n

    def observe(self, x, censored, tau):
        pass


class StaticCutoff(FullSync):
    """The same cutoff in every iteration (the fixed-backup-workers scheme Sec. 2 cites)."""

    def __init__(self, n, c):
        super().__init__(n)
        self.c = int(c)

    def decide(self):
        return self.c


class OrderCutoff:
    """The "order" comparison method of Sec. 4: iid normal run-times with the mean and spread of the
    last `lag` observed vectors, expected order statistics by eq. (4), same argmax rule.
    READING: a cut-off worker enters the window with its censoring time (the paper does not say)."""

    def __init__(self, n, lag):
        self.n, self.lag, self.window = n, lag, []

    def decide(self):
        if len(self.window) < self.lag:
            return self.n
        w = np.asarray(self.window[-self.lag:], dtype=np.float64)
        return binding.cutoff_elfving(self.n, float(w.mean()), float(w.std()))["cstar"]

    def observe(self, x, censored, tau):
        self.window.append(np.where(censored, tau, x))
        del self.window[:-self.lag]


class OraclePredictor:
    """The paper's predictor on the CPU oracle: decide from S sampled run-time vectors, then complete
    the censored observation from those same samples (Sec. 4.2) and push it into the window."""

    def __init__(self, cfg, blob, samples, noise, seed=0):
        self.cfg, self.S, self.noise = cfg, samples, noise
        self.model = binding.OracleModel(cfg, blob)
        self.rng = np.random.default_rng(seed)
        self.step, self.pushed, self.last = 0, 0, None

    def decide(self):
        self.step += 1
        if self.pushed < self.cfg.lag:
            self.last = None
            return self.cfg.n_workers
        eq, ez, ex = self.noise(self.step)
        self.last = self.model.sample_runtimes(eq, ez, ex).astype(np.float32)
        return binding.cutoff_select(self.last, want_sorted=False, want_perm=False)["cstar"]

    def observe(self, x, censored, tau):
        x = np.asarray(x, dtype=np.float32)
        if censored.any():
            u = self.rng.random(x.size).astype(np.float32)
            x, _ = binding.impute_censored(self.last, x, censored.astype(np.uint8), np.float32(tau), u)
        self.model.filter_step(x)
        self.pushed += 1


class LeastSquares:
    """A synthetic objective for step 4: F(theta) = mean_i (a_i . theta - y_i)^2 / 2 over M seeded
    records; a worker's gradient is the mean over b records drawn with replacement."""

    def __init__(self, n_workers, dim=16, records=4096, batch=32, lr=0.1, seed=0):
        g = np.random.default_rng(seed)
        self.A = g.standard_normal((records, dim))
        self.y = self.A @ g.standard_normal(dim) + 0.1 * g.standard_normal(records)
        self.theta = np.zeros(dim)
        self.n, self.b, self.lr, self.g = n_workers, batch, lr, g

    def loss(self):
        r = self.A @ self.theta - self.y
        return 0.5 * float(r @ r) / r.size

    def gradients(self):
        """[n][dim]: what each worker would send for the current theta."""
        idx = self.g.integers(0, self.y.size, (self.n, self.b))
        r = np.einsum("wbd,d->wb", self.A[idx], self.theta) - self.y[idx]
        return np.einsum("wb,wbd->wd", r, self.A[idx]) / self.b

    def apply(self, grads, bits, c):
        masked = grads * np.unpackbits(bits, count=self.n)[:, None]   # non-participants zero their gradients
        self.theta = self.theta - self.lr * masked.sum(axis=0) / c     # all-reduce, then the local update


@dataclass
class Run:
    cutoffs: List[int] = field(default_factory=list)
    tau: List[float] = field(default_factory=list)
    clock: List[float] = field(default_factory=list)      # wall-clock at the END of each iteration
    bits: List[np.ndarray] = field(default_factory=list)  # participants, packed as np.packbits does
    loss: List[float] = field(default_factory=list)

    @property
    def gradients_per_second(self):
        return float(np.sum(self.cutoffs) / self.clock[-1])


def simulate(trace, policy, overhead: float = 0.0, objective: Optional[LeastSquares] = None) -> Run:
    """Run Alg. 1's server loop over trace [T][N] (seconds).  `overhead` seconds are added to every
    iteration (decision, update and broadcast)."""
    trace = np.asarray(trace)
    T, n = trace.shape
    run, clock = Run(), 0.0
    for t in range(T):
        c = int(policy.decide())
        if not 1 <= c <= n:
            raise ValueError(f"iteration {t}: cutoff {c} outside [1, {n}]")
        grads = objective.gradients() if objective is not None else None
        queue = [(clock + float(trace[t, w]), w) for w in range(n)]
        heapq.heapify(queue)
        took = np.zeros(n, dtype=bool)
        finish = clock
        for _ in range(c):
            finish, w = heapq.heappop(queue)
            took[w] = True
        last = max((w for w in range(n) if took[w]), key=lambda w: (float(trace[t, w]), w))
        tau = float(trace[t, last])          # the run-time the c-th message reported
        bits = np.packbits(took)
        if objective is not None:
            objective.apply(grads, bits, c)
            run.loss.append(objective.loss())
        clock = finish + overhead
        policy.observe(np.where(took, trace[t], tau), ~took, tau)
        run.cutoffs.append(c)
        run.tau.append(tau)
        run.clock.append(clock)
        run.bits.append(bits)
    return run
