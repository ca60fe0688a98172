"""Compressed-activation convolution training step for AMD MI355X (gfx950).

The compute lives in hand-written HIP kernels behind a C ABI (include/cac.h);
this package is the thin Python binding plus seeded input generators.  The
native library is loaded on first use and its absence is an error: there is no
CPU fallback.
"""
from . import synth  # noqa: F401

__all__ = ["synth", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
