"""MI355X-native brick SpMM (C = A.B, A sparse CSR -> 16-row panels of 16x4 bricks).

`workloads` (input generators) imports nothing native.  The C-ABI binding is
loaded on first use of any other attribute and raises if the HIP library has
not been built.
"""
import importlib

__all__ = ["workloads", "binding"]


def __getattr__(name):
    if name in ("workloads", "binding"):
        return importlib.import_module(f"{__name__}.{name}")
    binding = importlib.import_module(f"{__name__}.binding")
    try:
        return getattr(binding, name)
    except AttributeError:
        raise AttributeError(f"module {__name__!r} has no attribute {name!r}") from None
