"""MI355X-native Cutoff-SGD run-time predictor (hand-written HIP behind a C ABI).

The binding in `api` loads `libcutoff_dkf.so` on first use and raises if it is
missing: there is no CPU fallback.
"""

__all__ = ["api"]


def __getattr__(name):
    if name == "api":
        import importlib

        return importlib.import_module(".api", __name__)
    raise AttributeError(name)
