"""int8 conv2d through a layout transformation + int8 MFMA on MI355X (gfx950).

`inputs` (seeded synthetic workloads) is importable without the HIP library;
everything else is a thin ctypes binding over the C-ABI in `include/conv2d_int8.h`
and is loaded on first use.
"""
from importlib import import_module

__all__ = ["inputs", "binding"]


def __getattr__(name):
    if name in __all__:
        return import_module(f"{__name__}.{name}")
    raise AttributeError(name)
