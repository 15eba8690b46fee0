"""bench.py's contract that can be checked without a GPU."""
import subprocess
import sys
from pathlib import Path

ROOT = Path(__file__).resolve().parents[1]


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, str(ROOT / "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_stage_work_matches_the_layer_sizes():
    sys.path.insert(0, str(ROOT))
    import bench
    import cluster_synth as synth

    cfg = synth.CONFIGS["medium"]
    w = bench.stage_work(cfg)
    S, N, L, Z, H, R = cfg.samples, cfg.n_workers, cfg.lag, cfg.z_dim, cfg.hidden, cfg.rnn_dim
    # guide: L steps of Z->R, R->Z, Z->Z; transition: two Z->H->Z branches, two Z->Z layers
    assert w[1][1] == 2.0 * S * (L * (Z * R + R * Z + Z * Z) + 2 * (Z * H + H * Z) + 2 * Z * Z)
    # emission: Z->H, H->N, N->H, H->N
    assert [w[s][1] for s in (2, 3, 4, 5)] == [2.0 * S * Z * H, 2.0 * S * H * N, 2.0 * S * N * H, 2.0 * S * H * N]
    assert w[8][1] == sum(w[s][1] for s in range(1, 6))
    # the fused kernel applies the N->H layer folded into an H x H one
    assert w[8][2] == w[8][1] - 2.0 * S * N * H + 2.0 * S * H * H
    assert w[6][:2] == ("hbm", 4.0 * S * N)
    # bf16: stage 4 is the folded layer, stage 5 both N-wide output layers; the algorithmic total is unchanged
    cfg = synth.CONFIGS["large_bf16"]
    w = bench.stage_work(cfg)
    S, N, H = cfg.samples, cfg.n_workers, cfg.hidden
    assert 3 not in w and w[4][1:] == (2.0 * S * N * H, 2.0 * S * H * H) and w[5][1] == w[5][2] == 2 * 2.0 * S * H * N
    assert sum(w[s][1] for s in (1, 2, 4, 5)) == w[8][1]
    assert abs(w[8][1] - 77.2e9) < 0.1e9  # the survey's figure for this configuration


def test_sort_compare_exchange_counts():
    sys.path.insert(0, str(ROOT))
    import bench

    # a bitonic network over n = 2^p keys has p (p + 1) / 2 stages of n / 2 compare-exchanges
    assert bench.sort_compare_exchanges(1, 8) == 4 * 6
    assert bench.sort_compare_exchanges(16384, 512) == 16384 * 256 * 45
    assert bench.sort_compare_exchanges(8192, 2048) == 8192 * 1024 * 66
    assert bench.sort_compare_exchanges(3, 158) == 3 * 128 * 36  # padded to 256 keys
