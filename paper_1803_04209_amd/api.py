"""ctypes binding of libcutoff_dkf.so: argument marshalling only.

Functions carry the names of the C entry points declared in
include/cutoff_dkf.h.  Device buffers are torch CUDA tensors (PyTorch is used
for device memory and streams, nothing else); every step of the predictor runs
inside the library's HIP kernels.  If the library has not been built, or no
GPU is present when a compute call is made, the call raises: there is no CPU
fallback.
"""
from __future__ import annotations

import ctypes as C
from pathlib import Path
from typing import Optional

import numpy as np

PKG = Path(__file__).resolve().parent
LIB_PATH = PKG / "libcutoff_dkf.so"

DKF_OK, DKF_WARMUP, CUTOFF_NO_ELIGIBLE = 0, 1, 2
DKF_EINVAL, DKF_ENOTREADY, DKF_EBADOBS, DKF_EHIP, DKF_ENOMEM, DKF_EBLOB, DKF_EUNSUPPORTED = -1, -2, -3, -4, -5, -6, -7
DKF_ESTALLED = -8
DKF_DTYPE_F32, DKF_DTYPE_BF16 = 0, 1
DKF_NUM_STAGES = 9
STAGE_NAMES = ["filter", "guide_transition", "emit_hidden", "emit_mean", "emit_scale_hidden",
               "emit_scale_draw", "sort_rank_sums", "means_argmax", "sampler_fused"]

EXPORTS = [
    "dkf_strerror", "dkf_last_hip_error", "dkf_blob_bytes", "dkf_load_weights", "dkf_free", "dkf_reset",
    "dkf_filter_step", "dkf_sample_runtimes", "cutoff_select", "cutoff_select_rate", "cutoff_select_workspace", "cutoff_select_static", "cutoff_select_static_max_workspace", "dkf_decide", "dkf_decide_trace",
    "dkf_check", "dkf_set_exchange_spin_limit", "dkf_decide_samples", "dkf_impute_censored", "dkf_impute_workspace", "cutoff_rank_spread", "cutoff_rank_spread_workspace", "dkf_get_state", "dkf_set_state", "dkf_set_sampler", "dkf_sampler_in_use", "dkf_decide_sorts_in_sampler", "dkf_timing_enable", "dkf_timing_read",
]


class DkfError(RuntimeError):
    def __init__(self, fn: str, code: int):
        self.code = code
        msg = _lib().dkf_strerror(code).decode()
        extra = f" (hipError {_lib().dkf_last_hip_error()})" if code == DKF_EHIP else ""
        super().__init__(f"{fn}: {msg}{extra} [{code}]")


class dkf_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_workers", "lag", "z_dim", "hidden", "rnn_dim", "mlp_dtype", "emit_mean_act", "max_samples")]


class dkf_stage_outputs(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("ctx", "z_last", "z_next", "emit_mean", "emit_sd")]


_handle = None


def _lib():
    """Load the shared library (raises if it has not been built)."""
    global _handle
    if _handle is not None:
        return _handle
    if not LIB_PATH.exists():
        raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_1803_04209_amd.build); "
                           "there is no CPU fallback")
    # PyTorch ships its own HIP runtime; load it first so that this library binds to the
    # same copy (two runtimes in one process do not see the device)
    import torch  # noqa: F401

    lib = C.CDLL(str(LIB_PATH))
    vp, i32, u64, sz, f32 = C.c_void_p, C.c_int32, C.c_uint64, C.c_size_t, C.c_float
    lib.dkf_strerror.restype = C.c_char_p
    lib.dkf_strerror.argtypes = [C.c_int]
    lib.dkf_last_hip_error.restype = C.c_int
    lib.dkf_blob_bytes.restype = sz
    lib.dkf_blob_bytes.argtypes = [C.POINTER(dkf_config)]
    lib.dkf_load_weights.argtypes = [C.POINTER(dkf_config), vp, sz, vp, C.POINTER(vp)]
    lib.dkf_free.argtypes = [vp]
    lib.dkf_reset.argtypes = [vp]
    lib.dkf_filter_step.argtypes = [vp, vp, vp]
    lib.dkf_sample_runtimes.argtypes = [vp, i32, vp, vp, vp, u64, vp, C.POINTER(dkf_stage_outputs), vp]
    lib.cutoff_select.argtypes = [vp, i32, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.cutoff_select_rate.argtypes = [vp, i32, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.cutoff_select_workspace.restype = sz
    lib.cutoff_select_workspace.argtypes = [i32, i32]
    lib.cutoff_select_static.argtypes = [vp, i32, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp]
    lib.cutoff_select_static_max_workspace.restype = sz
    lib.cutoff_select_static_max_workspace.argtypes = []
    lib.dkf_decide.argtypes = [vp, vp, i32, vp, vp, vp, u64, C.POINTER(i32), vp]
    lib.dkf_decide_trace.argtypes = [vp, vp, i32, i32, vp, vp, vp, u64, vp, vp, vp, vp]
    lib.dkf_check.argtypes = [vp, vp]
    lib.dkf_set_exchange_spin_limit.argtypes = [vp, i32]
    lib.dkf_decide_samples.restype = vp
    lib.dkf_decide_samples.argtypes = [vp]
    lib.dkf_impute_censored.argtypes = [vp, i32, i32, vp, vp, f32, vp, vp, vp, vp, sz, vp]
    lib.dkf_impute_workspace.restype = sz
    lib.dkf_impute_workspace.argtypes = [i32, i32]
    lib.cutoff_rank_spread.argtypes = [vp, i32, i32, vp, vp, vp, sz, vp]
    lib.cutoff_rank_spread_workspace.restype = sz
    lib.cutoff_rank_spread_workspace.argtypes = [i32, i32]
    lib.dkf_get_state.argtypes = [vp, vp, C.POINTER(sz)]
    lib.dkf_set_state.argtypes = [vp, vp, sz]
    lib.dkf_set_sampler.argtypes = [C.c_void_p, C.c_int32]
    lib.dkf_sampler_in_use.argtypes = [C.c_void_p, C.c_int32]
    lib.dkf_decide_sorts_in_sampler.argtypes = [C.c_void_p, C.c_int32]
    lib.dkf_timing_enable.argtypes = [C.c_uint32]
    lib.dkf_timing_read.argtypes = [i32, C.POINTER(i32), C.POINTER(C.c_double)]
    _handle = lib
    return lib


def _torch():
    import torch

    if not torch.cuda.is_available():
        raise RuntimeError("no GPU visible: the predictor runs only on the HIP path")
    return torch


def _stream_ptr(stream=None) -> int:
    torch = _torch()
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _dev(t, dtype, shape=None, name="tensor") -> Optional[int]:
    """Device pointer of a contiguous CUDA tensor (None passes NULL)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype:
        raise ValueError(f"{name}: need a contiguous CUDA tensor of {dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: shape {tuple(t.shape)}, expected {tuple(shape)}")
    return t.data_ptr()


def _check(fn: str, rc: int) -> int:
    if rc < 0:
        raise DkfError(fn, rc)
    return rc


def make_config(cfg, max_samples=None, emit_mean_act=0, mlp_dtype=None) -> dkf_config:
    """dkf_config from an object with n_workers, lag, z_dim, hidden, rnn_dim, samples, mlp_dtype attributes."""
    if mlp_dtype is None:
        mlp_dtype = DKF_DTYPE_BF16 if getattr(cfg, "mlp_dtype", "f32") == "bf16" else DKF_DTYPE_F32
    return dkf_config(cfg.n_workers, cfg.lag, cfg.z_dim, cfg.hidden, cfg.rnn_dim, int(mlp_dtype),
                      int(emit_mean_act), int(max_samples if max_samples is not None else cfg.samples))


# ---- the C entry points, same names ---------------------------------------------------

def dkf_blob_bytes(config: dkf_config) -> int:
    return int(_lib().dkf_blob_bytes(C.byref(config)))


def dkf_load_weights(config: dkf_config, blob: np.ndarray, stream=None) -> int:
    """Returns the opaque model handle (an int)."""
    _torch()
    raw = np.ascontiguousarray(blob).view(np.uint8)
    out = C.c_void_p()
    _check("dkf_load_weights",
           _lib().dkf_load_weights(C.byref(config), raw.ctypes.data, raw.size, _stream_ptr(stream), C.byref(out)))
    return out.value


def dkf_free(model: int) -> None:
    _check("dkf_free", _lib().dkf_free(model))


def dkf_reset(model: int) -> None:
    _check("dkf_reset", _lib().dkf_reset(model))


def dkf_filter_step(model: int, x_obs: np.ndarray, stream=None) -> int:
    x = np.ascontiguousarray(x_obs, dtype=np.float32)
    return _check("dkf_filter_step", _lib().dkf_filter_step(model, x.ctypes.data, _stream_ptr(stream)))


def dkf_sample_runtimes(model: int, S: int, eps_q, eps_z, eps_x, seed: int, out_samples,
                        stages: Optional[dkf_stage_outputs] = None, stream=None) -> int:
    torch = _torch()
    f = torch.float32
    return _check("dkf_sample_runtimes", _lib().dkf_sample_runtimes(
        model, S, _dev(eps_q, f, name="eps_q"), _dev(eps_z, f, name="eps_z"), _dev(eps_x, f, name="eps_x"),
        int(seed), _dev(out_samples, f, name="out_samples"),
        C.byref(stages) if stages is not None else None, _stream_ptr(stream)))


def cutoff_select_workspace(S: int, N: int) -> int:
    return int(_lib().cutoff_select_workspace(S, N))


def cutoff_select(samples, c_min: int, c_max: int, t_floor: float, out_sorted, out_perm, out_mean, out_omega,
                  out_cstar, workspace, stream=None) -> int:
    torch = _torch()
    S, N = samples.shape
    return _check("cutoff_select", _lib().cutoff_select(
        _dev(samples, torch.float32, name="samples"), S, N, c_min, c_max, float(t_floor),
        _dev(out_sorted, torch.float32, (S, N), "out_sorted"), _dev(out_perm, torch.int32, (S, N), "out_perm"),
        _dev(out_mean, torch.float32, (N,), "out_mean"), _dev(out_omega, torch.float32, (N,), "out_omega"),
        _dev(out_cstar, torch.int32, (2,), "out_cstar"), _dev(workspace, torch.uint8, name="workspace"),
        workspace.numel(), _stream_ptr(stream)))


def cutoff_select_rate(samples, c_min: int, c_max: int, t_floor: float, out_sorted, out_perm, out_rate, out_omega,
                       out_cstar, workspace, stream=None) -> int:
    torch = _torch()
    S, N = samples.shape
    return _check("cutoff_select_rate", _lib().cutoff_select_rate(
        _dev(samples, torch.float32, name="samples"), S, N, c_min, c_max, float(t_floor),
        _dev(out_sorted, torch.float32, (S, N), "out_sorted"), _dev(out_perm, torch.int32, (S, N), "out_perm"),
        _dev(out_rate, torch.float32, (N,), "out_rate"), _dev(out_omega, torch.float32, (N,), "out_omega"),
        _dev(out_cstar, torch.int32, (2,), "out_cstar"), _dev(workspace, torch.uint8, name="workspace"),
        workspace.numel(), _stream_ptr(stream)))


def cutoff_select_static_max_workspace() -> int:
    return int(_lib().cutoff_select_static_max_workspace())


def cutoff_select_static(samples, c_min: int, c_max: int, t_floor: float, out_sorted, out_perm, out_mean, out_omega,
                         out_cstar, stream=None) -> int:
    torch = _torch()
    S, N = samples.shape
    return _check("cutoff_select_static", _lib().cutoff_select_static(
        _dev(samples, torch.float32, name="samples"), S, N, c_min, c_max, float(t_floor),
        _dev(out_sorted, torch.float32, (S, N), "out_sorted"), _dev(out_perm, torch.int32, (S, N), "out_perm"),
        _dev(out_mean, torch.float32, (N,), "out_mean"), _dev(out_omega, torch.float32, (N,), "out_omega"),
        _dev(out_cstar, torch.int32, (2,), "out_cstar"), _stream_ptr(stream)))


def cutoff_rank_spread_workspace(S: int, N: int) -> int:
    return int(_lib().cutoff_rank_spread_workspace(S, N))


def cutoff_rank_spread(sorted_rows, mean, out_sd, workspace, stream=None) -> int:
    torch = _torch()
    S, N = sorted_rows.shape
    return _check("cutoff_rank_spread", _lib().cutoff_rank_spread(
        _dev(sorted_rows, torch.float32, name="sorted"), S, N, _dev(mean, torch.float32, (N,), "mean"),
        _dev(out_sd, torch.float32, (N,), "out_sd"), _dev(workspace, torch.uint8, name="workspace"),
        workspace.numel(), _stream_ptr(stream)))


def dkf_decide(model: int, x_obs: np.ndarray, S: int, eps_q, eps_z, eps_x, seed: int = 0, stream=None):
    """Returns (c*, status)."""
    torch = _torch()
    f = torch.float32
    x = np.ascontiguousarray(x_obs, dtype=np.float32)
    c = C.c_int32(0)
    rc = _check("dkf_decide", _lib().dkf_decide(
        model, x.ctypes.data, S, _dev(eps_q, f, name="eps_q"), _dev(eps_z, f, name="eps_z"),
        _dev(eps_x, f, name="eps_x"), int(seed), C.byref(c),
        _stream_ptr(stream) if stream is not None else None))
    return int(c.value), rc


def dkf_decide_trace(model: int, trace: np.ndarray, S: int, eps_q, eps_z, eps_x, seed: int = 0, stream=None):
    """One dkf_decide per row of `trace` ([T][N]) inside the library.  Returns (c* int32[T], status int32[T],
    latency in microseconds float32[T])."""
    torch = _torch()
    f = torch.float32
    x = np.ascontiguousarray(trace, dtype=np.float32)
    T = int(x.shape[0])
    c, st, lat = np.zeros(T, np.int32), np.zeros(T, np.int32), np.zeros(T, np.float32)
    _check("dkf_decide_trace", _lib().dkf_decide_trace(
        model, x.ctypes.data, T, S, _dev(eps_q, f, name="eps_q"), _dev(eps_z, f, name="eps_z"),
        _dev(eps_x, f, name="eps_x"), int(seed), c.ctypes.data, st.ctypes.data, lat.ctypes.data,
        _stream_ptr(stream) if stream is not None else None))
    return c, st, lat


def dkf_check(model: int, stream=None) -> int:
    """DKF_OK, or DKF_ESTALLED (returned, not raised) if the last filter step gave up."""
    rc = _lib().dkf_check(model, _stream_ptr(stream))
    return rc if rc == DKF_ESTALLED else _check("dkf_check", rc)


def dkf_set_exchange_spin_limit(model: int, polls: int) -> None:
    _check("dkf_set_exchange_spin_limit", _lib().dkf_set_exchange_spin_limit(model, polls))


def dkf_impute_workspace(S: int, N: int) -> int:
    return int(_lib().dkf_impute_workspace(S, N))


def dkf_impute_censored(samples, x_obs, censored, tau: float, u, x_full, n_exceed, workspace, stream=None) -> int:
    torch = _torch()
    S, N = samples.shape
    f = torch.float32
    return _check("dkf_impute_censored", _lib().dkf_impute_censored(
        _dev(samples, f, name="samples"), S, N, _dev(x_obs, f, (N,), "x_obs"),
        _dev(censored, torch.uint8, (N,), "censored"), float(tau), _dev(u, f, (N,), "u"),
        _dev(x_full, f, (N,), "x_full"), _dev(n_exceed, torch.int32, (N,), "n_exceed"),
        _dev(workspace, torch.uint8, name="workspace"), workspace.numel(), _stream_ptr(stream)))


def dkf_get_state(model: int) -> bytes:
    n = C.c_size_t(0)
    _check("dkf_get_state", _lib().dkf_get_state(model, None, C.byref(n)))
    buf = (C.c_char * n.value)()
    _check("dkf_get_state", _lib().dkf_get_state(model, buf, C.byref(n)))
    return bytes(buf)


def dkf_set_state(model: int, state: bytes) -> None:
    _check("dkf_set_state", _lib().dkf_set_state(model, state, len(state)))


SAMPLER_AUTO, SAMPLER_WAVE16, SAMPLER_WAVE4, SAMPLER_STAGED, SAMPLER_SPLIT = 0, 1, 2, 3, 4


def dkf_set_sampler(handle, variant: int) -> None:
    _check("dkf_set_sampler", _lib().dkf_set_sampler(handle, variant))


def dkf_sampler_in_use(handle, S: int) -> int:
    return _check("dkf_sampler_in_use", _lib().dkf_sampler_in_use(handle, int(S)))


def dkf_decide_sorts_in_sampler(handle, S: int) -> bool:
    return bool(_check("dkf_decide_sorts_in_sampler", _lib().dkf_decide_sorts_in_sampler(handle, int(S))))


def dkf_timing_enable(stage_mask: int) -> None:
    _check("dkf_timing_enable", _lib().dkf_timing_enable(stage_mask))


def dkf_timing_read(stage: int):
    """(launches, total milliseconds) recorded for one stage since the last read."""
    n, ms = C.c_int32(0), C.c_double(0.0)
    _check("dkf_timing_read", _lib().dkf_timing_read(stage, C.byref(n), C.byref(ms)))
    return int(n.value), float(ms.value)


# ---- small conveniences on top (still marshalling only) -----------------------------------

class Predictor:
    """Owns one dkf_model handle and the torch buffers its calls need."""

    def __init__(self, cfg, blob: np.ndarray, max_samples=None, emit_mean_act=0, mlp_dtype=None):
        self.cfg = cfg
        self.config = make_config(cfg, max_samples, emit_mean_act, mlp_dtype)
        self.handle = dkf_load_weights(self.config, blob)

    def close(self, _free=dkf_free):
        if getattr(self, "handle", None):
            handle, self.handle = self.handle, None
            _free(handle)

    def __del__(self):
        try:
            self.close()
        except Exception:  # interpreter shutdown: the library may already be gone
            pass

    def set_sampler(self, variant: int) -> None:
        dkf_set_sampler(self.handle, variant)

    def sampler_in_use(self, S: int) -> int:
        return dkf_sampler_in_use(self.handle, S)

    def decide_sorts_in_sampler(self, S: int) -> bool:
        return dkf_decide_sorts_in_sampler(self.handle, S)

    def reset(self):
        dkf_reset(self.handle)

    def filter_step(self, x_obs) -> int:
        return dkf_filter_step(self.handle, x_obs)

    def sample_runtimes(self, eps_q=None, eps_z=None, eps_x=None, stages: bool = False, out=None, S=None, seed=0):
        """With the three noise tensors: use them.  With none: the library draws its own from `seed` for S samples."""
        torch = _torch()
        cfg = self.cfg
        S = int(eps_z.shape[0] if eps_z is not None else S)
        dev = eps_z.device if eps_z is not None else torch.device("cuda")
        out = torch.empty((S, cfg.n_workers), dtype=torch.float32, device=dev) if out is None else out
        st, tensors = None, None
        if stages:
            tensors = dict(
                ctx=torch.empty((cfg.lag, cfg.rnn_dim), dtype=torch.float32, device=dev),
                z_T=torch.empty((S, cfg.z_dim), dtype=torch.float32, device=dev),
                z_next=torch.empty((S, cfg.z_dim), dtype=torch.float32, device=dev),
                emit_mean=torch.empty((S, cfg.n_workers), dtype=torch.float32, device=dev),
                emit_sd=torch.empty((S, cfg.n_workers), dtype=torch.float32, device=dev),
            )
            st = dkf_stage_outputs(tensors["ctx"].data_ptr(), tensors["z_T"].data_ptr(),
                                   tensors["z_next"].data_ptr(), tensors["emit_mean"].data_ptr(),
                                   tensors["emit_sd"].data_ptr())
        dkf_sample_runtimes(self.handle, S, eps_q, eps_z, eps_x, seed, out, st)
        return (out, tensors) if stages else out

    def decide(self, x_obs, S, eps_q=None, eps_z=None, eps_x=None, seed=0):
        return dkf_decide(self.handle, x_obs, S, eps_q, eps_z, eps_x, seed)

    def decide_trace(self, trace, S, eps_q=None, eps_z=None, eps_x=None, seed=0):
        return dkf_decide_trace(self.handle, trace, S, eps_q, eps_z, eps_x, seed)

    def decide_samples(self, S):
        """Copy of the [S][N] samples behind the last decide()."""
        torch = _torch()
        ptr = _lib().dkf_decide_samples(self.handle)

        class _View:  # zero-copy description of library-owned device memory
            __cuda_array_interface__ = {"shape": (S, self.cfg.n_workers), "typestr": "<f4",
                                        "data": (int(ptr), False), "version": 2}

        torch.cuda.synchronize()
        return torch.as_tensor(_View(), device="cuda").clone()

    def get_state(self) -> bytes:
        return dkf_get_state(self.handle)

    def set_state(self, state: bytes):
        dkf_set_state(self.handle, state)


def impute_censored(samples, x_obs, censored, tau, u):
    """Allocate outputs + workspace, call dkf_impute_censored, return (x_full, n_exceed) tensors."""
    torch = _torch()
    S, N = samples.shape
    dev = samples.device
    ws = torch.empty(dkf_impute_workspace(S, N), dtype=torch.uint8, device=dev)
    x_full = torch.empty(N, dtype=torch.float32, device=dev)
    n_exceed = torch.empty(N, dtype=torch.int32, device=dev)
    dkf_impute_censored(samples, x_obs, censored, tau, u, x_full, n_exceed, ws)
    return x_full, n_exceed


def rank_spread(sorted_rows, mean):
    """Allocate output + workspace, call cutoff_rank_spread, return the sd tensor [N]."""
    torch = _torch()
    S, N = sorted_rows.shape
    ws = torch.empty(max(cutoff_rank_spread_workspace(S, N), 256), dtype=torch.uint8, device=sorted_rows.device)
    sd = torch.empty(N, dtype=torch.float32, device=sorted_rows.device)
    cutoff_rank_spread(sorted_rows, mean, sd, ws)
    return sd


def select_cutoff(samples, c_min=1, c_max=None, t_floor=0.0, want_sorted=False, want_perm=False, rate=False):
    """Allocate outputs + workspace, call cutoff_select (or, with rate=True, cutoff_select_rate, whose
    out_rate then sits under the key "mean"), return a dict of tensors and ints."""
    torch = _torch()
    S, N = samples.shape
    c_max = N if c_max is None else c_max
    dev = samples.device
    ws_bytes = cutoff_select_workspace(S, N)
    if ws_bytes == 0:
        raise DkfError("cutoff_select_workspace", DKF_EUNSUPPORTED)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    srt = torch.empty((S, N), dtype=torch.float32, device=dev) if want_sorted else None
    perm = torch.empty((S, N), dtype=torch.int32, device=dev) if want_perm else None
    mean = torch.empty(N, dtype=torch.float32, device=dev)
    omega = torch.empty(N, dtype=torch.float32, device=dev)
    cstar = torch.zeros(2, dtype=torch.int32, device=dev)
    (cutoff_select_rate if rate else cutoff_select)(samples, c_min, c_max, t_floor, srt, perm, mean, omega, cstar, ws)
    c = cstar.cpu()
    return dict(cstar=int(c[0]), status=int(c[1]), mean=mean, omega=omega, sorted=srt, perm=perm)
