"""MI355X-native HALO low-precision linear layer (hand-written HIP kernels behind a C ABI).

`inputs`  : seeded synthetic tensors (no method arithmetic).
`binding` : ctypes marshalling onto libhalo.so; same names as include/halo.h.
"""
from importlib import import_module

__all__ = ["inputs", "binding", "build"]


def build(verbose: bool = False) -> str:
    """Compile libhalo.so in-tree (hipcc, gfx950)."""
    from . import _build
    return _build.build(verbose=verbose)


def __getattr__(name):
    if name in ("inputs", "binding"):
        return import_module("." + name, __name__)
    raise AttributeError(name)
