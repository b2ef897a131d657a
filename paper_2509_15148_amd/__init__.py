"""MI355X-native ATTS hot path: target-model scoring of shared-prefix drafts, online conformal
calibration and ordinal classification, as a C-ABI HIP library (libatts.so) plus a thin ctypes
binding (paper_2509_15148_amd.binding).  See include/atts.h for the contract of every entry point.

The binding is imported on first attribute access, so that `python -m paper_2509_15148_amd.build`
can run before the library exists; using anything else without a built library raises ImportError.
"""
import importlib

_BINDING = None


def __getattr__(name):
    global _BINDING
    if _BINDING is None:
        _BINDING = importlib.import_module(".binding", __name__)
    try:
        return getattr(_BINDING, name)
    except AttributeError:
        raise AttributeError(f"module {__name__!r} has no attribute {name!r}") from None
