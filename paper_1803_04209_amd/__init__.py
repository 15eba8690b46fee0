"""MI355X-native Cutoff-SGD run-time predictor (hand-written HIP behind a C ABI).

`synth` (seeded synthetic inputs) imports without the compiled library; the
binding in `api` loads `libcutoff_dkf.so` on first use and raises if it is
missing: there is no CPU fallback.
"""
from . import synth  # noqa: F401

__all__ = ["synth", "api"]


def __getattr__(name):
    if name == "api":
        import importlib

        return importlib.import_module(".api", __name__)
    raise AttributeError(name)
