"""GRASS structured-sparse gradient step on AMD MI355X (gfx950).

`grass` (the ctypes binding of the HIP library) is loaded on first use so that
importing the package, e.g. for `workloads`, does not need the built library.
"""
import importlib

__all__ = ["grass", "workloads"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
