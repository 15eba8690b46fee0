"""CPU oracle of the Cutoff-SGD predictor: test infrastructure, not product code.

Thin ctypes binding over `cutoff_oracle.c` (double precision, plain loops).
Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package; the GPU library never does.
"""
from .binding import (  # noqa: F401
    OracleModel,
    build,
    cutoff_elfving,
    cutoff_select,
    cutoff_select_rate,
    elfving_mean,
    fill_normal,
    impute_censored,
    make_noise,
    philox4x32_10,
    rank_spread,
    round_bf16,
    num_threads,
    set_threads,
    trace_throughput,
    NO_ELIGIBLE,
    OK,
    WARMUP,
)
