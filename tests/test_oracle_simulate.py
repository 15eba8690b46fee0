"""Pins of the discrete-event simulation of Alg. 1's server loop — CPU only.

The event-queue simulation is checked against what the loop must give in closed form: sums of
order statistics of the trace rows (computed here by sorting, and by the C oracle's own
throughput routine), the paper's 10 s / 8 s example, exact participant sets, and gradient steps
that reduce to plain gradient descent.
"""
import numpy as np
import pytest

import oracle
from oracle import simulate as sim
import cluster_synth as synth


def test_full_sync_and_static_cutoffs_are_sums_of_order_statistics():
    cfg = synth.CONFIGS["tiny"]
    trace = synth.make_trace(cfg, 80)
    srt = np.sort(trace.astype(np.float64), axis=1)
    n = cfg.n_workers
    run = sim.simulate(trace, sim.FullSync(n))
    assert np.allclose(run.clock, np.cumsum(srt[:, -1]), rtol=1e-12)
    assert abs(run.gradients_per_second - oracle.trace_throughput(trace, np.full(80, n))[1]) < 1e-9
    for c in (1, 5, n - 1):
        run = sim.simulate(trace, sim.StaticCutoff(n, c), overhead=0.25)
        assert np.allclose(run.clock, np.cumsum(srt[:, c - 1] + 0.25), rtol=1e-12)
        assert np.allclose(run.tau, srt[:, c - 1], rtol=0, atol=0)
        got = np.sum(run.cutoffs) / (run.clock[-1] - 0.25 * 80)
        assert abs(got - oracle.trace_throughput(trace, np.full(80, c))[0]) < 1e-9 * got


def test_papers_ten_and_eight_second_example():
    n = 12
    row = np.full(n, 5.0, dtype=np.float32)
    row[3], row[7] = 10.0, 8.0
    trace = np.tile(row, (4, 1))
    sync = sim.simulate(trace, sim.FullSync(n))
    drop = sim.simulate(trace, sim.StaticCutoff(n, n - 1))
    assert drop.clock[-1] == pytest.approx(0.8 * sync.clock[-1], rel=1e-12)   # 20 % less wall-clock
    took = np.unpackbits(drop.bits[0], count=n).astype(bool)
    assert not took[3] and took.sum() == n - 1


def test_participants_are_the_c_fastest_with_ties_in_worker_order():
    trace = np.array([[3.0, 1.0, 2.0, 1.0, 2.0, 9.0]], dtype=np.float32)
    for c, want in [(1, [1]), (2, [1, 3]), (3, [1, 2, 3]), (4, [1, 2, 3, 4]), (6, [0, 1, 2, 3, 4, 5])]:
        run = sim.simulate(trace, sim.StaticCutoff(6, c))
        took = np.flatnonzero(np.unpackbits(run.bits[0], count=6))
        assert took.tolist() == want
        assert run.tau[0] == np.sort(trace[0])[c - 1]


class Recorder(sim.StaticCutoff):
    def __init__(self, n, c):
        super().__init__(n, c)
        self.seen = []

    def observe(self, x, censored, tau):
        self.seen.append((np.array(x), np.array(censored), tau))


def test_the_server_never_sees_a_dropped_workers_time():
    cfg = synth.CONFIGS["tiny"]
    trace = synth.make_trace(cfg, 10)
    pol = Recorder(cfg.n_workers, 11)
    sim.simulate(trace, pol)
    for t, (x, cens, tau) in enumerate(pol.seen):
        assert cens.sum() == cfg.n_workers - 11
        assert np.array_equal(x[~cens], trace[t][~cens]) and np.all(x[cens] == tau)
        assert np.all(trace[t][cens] >= tau) and np.all(trace[t][~cens] <= tau)


def test_out_of_range_cutoff_is_an_error():
    with pytest.raises(ValueError):
        sim.simulate(np.ones((2, 4), dtype=np.float32), sim.StaticCutoff(4, 5))
    with pytest.raises(ValueError):
        sim.simulate(np.ones((2, 4), dtype=np.float32), sim.StaticCutoff(4, 0))


def test_masked_update_is_the_mean_over_participants():
    n = 8
    obj = sim.LeastSquares(n, dim=5, records=64, batch=64, lr=0.3, seed=1)
    theta0 = obj.theta.copy()
    grads = np.random.default_rng(0).standard_normal((n, 5))
    took = np.array([1, 0, 1, 1, 0, 0, 1, 0], dtype=bool)
    obj.apply(grads, np.packbits(took), int(took.sum()))
    assert np.allclose(obj.theta, theta0 - 0.3 * grads[took].mean(axis=0), rtol=1e-14)
    # identical worker gradients: any cutoff gives the plain gradient-descent step
    obj2 = sim.LeastSquares(n, dim=5, records=64, batch=64, lr=0.3, seed=1)
    same = np.tile(grads[0], (n, 1))
    obj2.apply(same, np.packbits(took), int(took.sum()))
    assert np.allclose(obj2.theta, -0.3 * grads[0], rtol=1e-14)


def test_worker_gradients_are_unbiased_for_the_full_gradient():
    obj = sim.LeastSquares(400, dim=6, records=512, batch=64, seed=2)
    obj.theta = np.random.default_rng(3).standard_normal(6)
    full = obj.A.T @ (obj.A @ obj.theta - obj.y) / obj.y.size
    g = obj.gradients()
    assert g.shape == (400, 6)
    assert np.allclose(g.mean(axis=0), full, atol=5 * g.std(axis=0).max() / np.sqrt(400))


def test_loss_falls_and_cutoff_reaches_it_in_less_simulated_time():
    cfg = synth.CONFIGS["tiny"]
    trace = synth.make_trace(cfg, 150)
    n = cfg.n_workers
    sync = sim.simulate(trace, sim.FullSync(n), objective=sim.LeastSquares(n, seed=5))
    cut = sim.simulate(trace, sim.StaticCutoff(n, n - 3), objective=sim.LeastSquares(n, seed=5))
    assert sync.loss[-1] < 0.05 * sync.loss[0] and cut.loss[-1] < 0.05 * cut.loss[0]
    target = 0.1 * sync.loss[0]
    t_sync = sync.clock[int(np.argmax(np.array(sync.loss) < target))]
    t_cut = cut.clock[int(np.argmax(np.array(cut.loss) < target))]
    assert t_cut < t_sync


def test_order_policy_warms_up_then_follows_elfving():
    n, lag = 16, 5
    trace = synth.make_trace(synth.CONFIGS["tiny"], 30)
    pol = sim.OrderCutoff(n, lag)
    run = sim.simulate(trace, pol)
    assert run.cutoffs[:lag] == [n] * lag
    # first decision after the warm-up: the window is the first `lag` full rows
    w = trace[:lag].astype(np.float64)
    assert run.cutoffs[lag] == oracle.cutoff_elfving(n, float(w.mean()), float(w.std()))["cstar"]


def test_oracle_predictor_policy_runs_alg1_with_censored_feedback():
    cfg = synth.CONFIGS["tiny"]
    trace = synth.make_trace(cfg, 40)
    pol = sim.OraclePredictor(cfg, synth.make_blob(cfg), samples=128,
                              noise=lambda step: synth.make_noise(cfg, samples=128, draw=step))
    run = sim.simulate(trace, pol)
    assert run.cutoffs[:cfg.lag] == [cfg.n_workers] * cfg.lag     # no prediction before the window is full
    assert all(1 <= c <= cfg.n_workers for c in run.cutoffs)
    assert min(run.cutoffs) < cfg.n_workers                        # it does cut workers off
    assert pol.pushed == 40
    # replaying the recorded cutoffs as a fixed schedule gives the same clock: decisions are the only coupling
    class Schedule(sim.FullSync):
        def __init__(self, cs):
            self.cs = iter(cs)
        def decide(self):
            return next(self.cs)
    again = sim.simulate(trace, Schedule(run.cutoffs))
    assert again.clock == run.clock and all(np.array_equal(a, b) for a, b in zip(again.bits, run.bits))
