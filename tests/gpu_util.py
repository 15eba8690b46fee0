"""Helpers shared by the GPU parity tests."""
import numpy as np


def rel_err(got, ref):
    """max |got - ref| / max(|ref|, rms(ref)): error relative to the tensor's own scale."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = np.sqrt(np.mean(ref ** 2)) if ref.size else 0.0
    denom = np.maximum(np.abs(ref), rms)
    denom = np.where(denom > 0, denom, 1.0)
    return float(np.max(np.abs(got - ref) / denom)) if ref.size else 0.0


def cstar_in_tie_band(c_gpu, oracle_result, rel=1e-6):
    """c* equal to the oracle's, or its oracle Omega within `rel` of the oracle maximum."""
    if c_gpu == oracle_result["cstar"]:
        return True
    om = oracle_result["omega"]
    best = om[oracle_result["cstar"] - 1]
    return np.isfinite(om[c_gpu - 1]) and om[c_gpu - 1] >= best - rel * abs(best)
