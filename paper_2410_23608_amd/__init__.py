"""MI355X (gfx950) implementation of the Select-and-Pack Attention hot path.

`spa` (the ctypes binding over libspa.so) is imported lazily so that the input
generators in `workloads` stay usable where the HIP library has not been built.
"""
import importlib

__all__ = ["spa", "workloads"]


def __getattr__(name):
    if name in ("spa", "workloads", "build"):
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
