"""ctypes binding for the C oracle (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "cutoff_oracle.c"
_LIB = _HERE / "libcutoff_oracle.so"

OK, WARMUP, NO_ELIGIBLE = 0, 1, 2


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_workers", "lag", "z_dim", "hidden", "rnn_dim", "emit_mean_act")]


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (plain C99 + OpenMP)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".tmp{os.getpid()}.so")
        subprocess.run(
            ["gcc", "-std=c99", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", str(tmp), str(_SRC), "-lm"],
            check=True,
        )
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = C.CDLL(str(_LIB))
    dp, fp, ip = C.POINTER(C.c_double), C.POINTER(C.c_float), C.POINTER(C.c_int32)
    lib.oracle_blob_bytes.restype = C.c_size_t
    lib.oracle_blob_bytes.argtypes = [C.POINTER(_Config)]
    lib.oracle_load_weights.restype = C.c_void_p
    lib.oracle_load_weights.argtypes = [C.POINTER(_Config), C.c_void_p, C.c_size_t]
    lib.oracle_free.argtypes = [C.c_void_p]
    lib.oracle_reset.argtypes = [C.c_void_p]
    lib.oracle_scale.restype = C.c_double
    lib.oracle_scale.argtypes = [C.c_void_p]
    lib.oracle_filter_step.argtypes = [C.c_void_p, dp]
    lib.oracle_encode_window.argtypes = [C.c_void_p, dp, dp]
    lib.oracle_sample_runtimes.argtypes = [C.c_void_p, C.c_int, ip, C.c_int, fp, fp, fp, dp, dp, dp, dp, dp]
    lib.oracle_set_mlp_bf16.argtypes = [C.c_void_p, C.c_int]
    lib.oracle_round_bf16.restype = C.c_double
    lib.oracle_round_bf16.argtypes = [C.c_double]
    lib.oracle_transition_terms.argtypes = [C.c_void_p, C.c_int, ip, C.c_int, fp, fp, fp, dp, dp, dp, dp, dp, dp, dp]
    lib.oracle_cutoff_select.argtypes = [dp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, dp, ip, dp, dp, ip]
    lib.oracle_cutoff_select_rate.argtypes = [dp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, dp, dp, ip]
    lib.oracle_cutoff_select_f32.argtypes = [fp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, dp, ip, dp, dp, ip]
    lib.oracle_predict_cutoff.argtypes = [C.c_void_p, C.c_int, fp, fp, fp, C.c_int, C.c_int, C.c_double, ip]
    lib.oracle_philox4x32_10.argtypes = [C.POINTER(C.c_uint32), C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
    lib.oracle_fill_normal.argtypes = [C.c_uint64, C.c_uint32, C.c_size_t, fp]
    u8 = C.POINTER(C.c_uint8)
    lib.oracle_impute_censored.argtypes = [fp, C.c_int, C.c_int, fp, u8, C.c_float, fp, fp, ip]
    lib.oracle_elfving_mean.restype = C.c_double
    lib.oracle_elfving_mean.argtypes = [C.c_int, C.c_int, C.c_double, C.c_double]
    lib.oracle_cutoff_elfving.argtypes = [C.c_int, C.c_double, C.c_double, C.c_int, C.c_int, C.c_double, dp, dp, ip]
    lib.oracle_trace_throughput.argtypes = [dp, C.c_int, C.c_int, ip, dp]
    lib.oracle_rank_spread.argtypes = [dp, C.c_int, C.c_int, dp, dp]
    lib.oracle_num_threads.restype = C.c_int
    lib.oracle_set_threads.argtypes = [C.c_int]
    _lib = lib
    return lib


def round_bf16(v: float) -> float:
    """Round to nearest-even bfloat16 (8 significant bits), returned as a double."""
    return float(_load().oracle_round_bf16(float(v)))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_threads(n: int) -> None:
    _load().oracle_set_threads(int(n))


def philox4x32_10(ctr, key):
    """Four output words of Philox4x32-10 for a 4-word counter and a 2-word key."""
    c = (C.c_uint32 * 4)(*ctr)
    k = (C.c_uint32 * 2)(*key)
    out = (C.c_uint32 * 4)()
    _load().oracle_philox4x32_10(c, k, out)
    return [int(v) for v in out]


def fill_normal(seed: int, tensor: int, shape) -> np.ndarray:
    """The sampler's own noise stream `tensor` (0 eps_q, 1 eps_z, 2 eps_x) for `seed`, fp32."""
    out = np.empty(shape, dtype=np.float32)
    _load().oracle_fill_normal(int(seed), int(tensor), out.size, _fp(out))
    return out


def make_noise(cfg, seed: int, samples=None):
    """(eps_q, eps_z, eps_x) exactly as the library draws them for `seed`."""
    S = int(samples if samples is not None else cfg.samples)
    return (fill_normal(seed, 0, (cfg.lag, S, cfg.z_dim)), fill_normal(seed, 1, (S, cfg.z_dim)),
            fill_normal(seed, 2, (S, cfg.n_workers)))


def _dp(a):
    return a.ctypes.data_as(C.POINTER(C.c_double)) if a is not None else None


def _fp(a):
    return a.ctypes.data_as(C.POINTER(C.c_float)) if a is not None else None


def _ip(a):
    return a.ctypes.data_as(C.POINTER(C.c_int32)) if a is not None else None


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


class OracleModel:
    """Weights + fixed-lag window of one predictor, on the CPU, in float64."""

    def __init__(self, cfg, blob: np.ndarray, emit_mean_act: int = 0, mlp_bf16: bool = False):
        """mlp_bf16: the sampler's mixed-precision mode (MLP matrices and their inputs rounded to bf16)."""
        lib = _load()
        self.cfg = cfg
        self._c = _Config(cfg.n_workers, cfg.lag, cfg.z_dim, cfg.hidden, cfg.rnn_dim, int(emit_mean_act))
        raw = np.ascontiguousarray(blob).view(np.uint8)
        self._h = lib.oracle_load_weights(C.byref(self._c), raw.ctypes.data, raw.size)
        if not self._h:
            raise ValueError("oracle_load_weights rejected the configuration or blob")
        if mlp_bf16:
            self.set_mlp_bf16(True)

    def set_mlp_bf16(self, on: bool) -> None:
        if _load().oracle_set_mlp_bf16(self._h, int(bool(on))) < 0:
            raise MemoryError("oracle_set_mlp_bf16")

    def close(self):
        if getattr(self, "_h", None):
            _load().oracle_free(self._h)
            self._h = None

    __del__ = close

    def reset(self):
        _load().oracle_reset(self._h)

    @property
    def scale(self) -> float:
        return float(_load().oracle_scale(self._h))

    def filter_step(self, x_obs) -> int:
        x = np.ascontiguousarray(x_obs, dtype=np.float64)
        assert x.shape == (self.cfg.n_workers,)
        rc = _load().oracle_filter_step(self._h, _dp(x))
        if rc < 0:
            raise ValueError(f"oracle_filter_step: error {rc}")
        return rc

    def encode_window(self):
        L, R = self.cfg.lag, self.cfg.rnn_dim
        hl, hr = np.empty((L, R)), np.empty((L, R))
        rc = _load().oracle_encode_window(self._h, _dp(hl), _dp(hr))
        if rc < 0:
            raise RuntimeError(f"oracle_encode_window: error {rc}")
        return hl, hr

    def sample_runtimes(self, eps_q, eps_z, eps_x, rows=None, stages: bool = False):
        """Samples [n][N] in seconds (float64); with stages=True also z_T, z_{T+1}, I, J."""
        cfg = self.cfg
        eps_q, eps_z, eps_x = _f32(eps_q), _f32(eps_z), _f32(eps_x)
        S = eps_z.shape[0]
        assert eps_q.shape == (cfg.lag, S, cfg.z_dim) and eps_z.shape == (S, cfg.z_dim)
        assert eps_x.shape == (S, cfg.n_workers)
        r = None if rows is None else np.ascontiguousarray(rows, dtype=np.int32)
        n = S if r is None else r.size
        x = np.empty((n, cfg.n_workers))
        zT = np.empty((n, cfg.z_dim)) if stages else None
        zn = np.empty((n, cfg.z_dim)) if stages else None
        mean = np.empty((n, cfg.n_workers)) if stages else None
        sd = np.empty((n, cfg.n_workers)) if stages else None
        rc = _load().oracle_sample_runtimes(self._h, S, _ip(r), n, _fp(eps_q), _fp(eps_z), _fp(eps_x),
                                            _dp(x), _dp(zT), _dp(zn), _dp(mean), _dp(sd))
        if rc < 0:
            raise RuntimeError(f"oracle_sample_runtimes: error {rc}")
        if stages:
            return x, dict(z_T=zT, z_next=zn, emit_mean=mean, emit_sd=sd)
        return x

    def transition_terms(self, eps_q, eps_z, eps_x, rows=None):
        """Inside of the gated transition per sample: gate_hidden [n][H] (before its ReLU), gate_pre
        (argument of the sigmoid), gate, lin, prop, G, Hs, each [n][Z]."""
        cfg = self.cfg
        eps_q, eps_z, eps_x = _f32(eps_q), _f32(eps_z), _f32(eps_x)
        S = eps_z.shape[0]
        assert eps_q.shape == (cfg.lag, S, cfg.z_dim) and eps_z.shape == (S, cfg.z_dim)
        r = None if rows is None else np.ascontiguousarray(rows, dtype=np.int32)
        n = S if r is None else r.size
        out = dict(gate_hidden=np.empty((n, cfg.hidden)))
        for k in ("gate_pre", "gate", "lin", "prop", "G", "Hs"):
            out[k] = np.empty((n, cfg.z_dim))
        rc = _load().oracle_transition_terms(self._h, S, _ip(r), n, _fp(eps_q), _fp(eps_z), _fp(eps_x),
                                             *[_dp(out[k]) for k in ("gate_hidden", "gate_pre", "gate", "lin", "prop", "G", "Hs")])
        if rc < 0:
            raise RuntimeError(f"oracle_transition_terms: error {rc}")
        return out

    def predict_cutoff(self, eps_q, eps_z, eps_x, c_min=1, c_max=None, t_floor=0.0):
        eps_q, eps_z, eps_x = _f32(eps_q), _f32(eps_z), _f32(eps_x)
        c_max = self.cfg.n_workers if c_max is None else c_max
        out = np.zeros(1, dtype=np.int32)
        rc = _load().oracle_predict_cutoff(self._h, eps_z.shape[0], _fp(eps_q), _fp(eps_z), _fp(eps_x),
                                           c_min, c_max, float(t_floor), _ip(out))
        if rc < 0:
            raise RuntimeError(f"oracle_predict_cutoff: error {rc}")
        return int(out[0]), rc


def cutoff_select(samples, c_min=1, c_max=None, t_floor=0.0, want_sorted=True, want_perm=True):
    """Sort rows, average ranks, Omega(c) = c / mean, argmax.  Returns a dict."""
    a = np.ascontiguousarray(samples)
    if a.ndim != 2:
        raise ValueError("samples must be [S][N]")
    S, N = a.shape
    c_max = N if c_max is None else c_max
    srt = np.empty((S, N)) if want_sorted else None
    perm = np.empty((S, N), dtype=np.int32) if want_perm else None
    mean, omega = np.empty(N), np.empty(N)
    cstar = np.zeros(1, dtype=np.int32)
    lib = _load()
    if a.dtype == np.float32:
        rc = lib.oracle_cutoff_select_f32(_fp(a), S, N, c_min, c_max, float(t_floor),
                                          _dp(srt), _ip(perm), _dp(mean), _dp(omega), _ip(cstar))
    else:
        a = np.ascontiguousarray(a, dtype=np.float64)
        rc = lib.oracle_cutoff_select(_dp(a), S, N, c_min, c_max, float(t_floor),
                                      _dp(srt), _ip(perm), _dp(mean), _dp(omega), _ip(cstar))
    if rc < 0:
        raise ValueError(f"oracle_cutoff_select: error {rc}")
    return dict(status=rc, cstar=int(cstar[0]), mean=mean, omega=omega, sorted=srt, perm=perm)


def cutoff_select_rate(samples, c_min=1, c_max=None, t_floor=0.0):
    """Omega(c) = mean_k c / x_(c)^(k) and its (largest) maximiser.  Returns a dict (rate, omega, cstar, status)."""
    a = np.ascontiguousarray(samples, dtype=np.float64)
    S, N = a.shape
    c_max = N if c_max is None else c_max
    rate, omega = np.empty(N), np.empty(N)
    cstar = np.zeros(1, dtype=np.int32)
    rc = _load().oracle_cutoff_select_rate(_dp(a), S, N, c_min, c_max, float(t_floor), _dp(rate), _dp(omega), _ip(cstar))
    if rc < 0:
        raise ValueError(f"oracle_cutoff_select_rate: error {rc}")
    return dict(status=rc, cstar=int(cstar[0]), rate=rate, omega=omega)


def impute_censored(samples, x_obs, censored, tau, u):
    """Fill in the run-times of dropped workers from the draws that exceed the censoring time.
    Returns (x_full float32[N], n_exceed int32[N])."""
    a = np.ascontiguousarray(samples, dtype=np.float32)
    S, N = a.shape
    xo = np.ascontiguousarray(x_obs, dtype=np.float32)
    cm = np.ascontiguousarray(censored, dtype=np.uint8)
    uu = np.ascontiguousarray(u, dtype=np.float32)
    out = np.empty(N, dtype=np.float32)
    cnt = np.empty(N, dtype=np.int32)
    rc = _load().oracle_impute_censored(_fp(a), S, N, _fp(xo), cm.ctypes.data_as(C.POINTER(C.c_uint8)), float(tau),
                                        _fp(uu), _fp(out), _ip(cnt))
    if rc < 0:
        raise ValueError(f"oracle_impute_censored: error {rc}")
    return out, cnt


def elfving_mean(j: int, n: int, mu: float, sigma: float) -> float:
    return float(_load().oracle_elfving_mean(j, n, mu, sigma))


def cutoff_elfving(n, mu, sigma, c_min=1, c_max=None, t_floor=0.0):
    c_max = n if c_max is None else c_max
    mean, omega = np.empty(n), np.empty(n)
    cstar = np.zeros(1, dtype=np.int32)
    rc = _load().oracle_cutoff_elfving(n, float(mu), float(sigma), c_min, c_max, float(t_floor), _dp(mean), _dp(omega),
                                       _ip(cstar))
    if rc < 0:
        raise ValueError(f"oracle_cutoff_elfving: error {rc}")
    return dict(status=rc, cstar=int(cstar[0]), mean=mean, omega=omega)


def trace_throughput(trace, cutoffs):
    """(achieved, full-sync, hindsight-best) gradients per second over a trace [T][N]."""
    tr = np.ascontiguousarray(trace, dtype=np.float64)
    T, N = tr.shape
    cs = np.ascontiguousarray(cutoffs, dtype=np.int32)
    out = np.empty(3)
    rc = _load().oracle_trace_throughput(_dp(tr), T, N, _ip(cs), _dp(out))
    if rc < 0:
        raise ValueError(f"oracle_trace_throughput: error {rc}")
    return tuple(float(v) for v in out)


def rank_spread(samples):
    """(mean [N], sd [N]) of every order statistic over the rows of samples [S][N] (divisor S)."""
    a = np.ascontiguousarray(samples, dtype=np.float64)
    if a.ndim != 2:
        raise ValueError("samples must be [S][N]")
    S, N = a.shape
    mean, sd = np.empty(N), np.empty(N)
    rc = _load().oracle_rank_spread(_dp(a), S, N, _dp(mean), _dp(sd))
    if rc < 0:
        raise ValueError(f"oracle_rank_spread: error {rc}")
    return mean, sd
