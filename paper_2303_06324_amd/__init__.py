"""MI355X-native preemptive daemon-kernel collectives (the hot path of arXiv 2303.06324).

The product is the HIP library `libdfx.so` (C ABI in include/dfx.h); this package is the thin
ctypes binding over it.  Using it requires the built library: there is no CPU path, and the first
access to any name of the binding raises ImportError when the library is missing.  The binding is
loaded at that first access rather than at import, so that `python -m paper_2303_06324_amd.build`
(the module that builds the library) can run in a tree that has none yet.
"""
import importlib

_SUBMODULES = ("binding", "build")


def __getattr__(name):
    if name in _SUBMODULES or name.startswith("__"):
        raise AttributeError(name)          # submodules are imported by the import system itself
    binding = importlib.import_module(".binding", __name__)     # raises ImportError without libdfx.so
    try:
        return getattr(binding, name)
    except AttributeError:
        raise AttributeError(f"module {__name__!r} has no attribute {name!r}") from None


def __dir__():
    binding = importlib.import_module(".binding", __name__)
    return sorted(set(globals()) | set(dir(binding)))
