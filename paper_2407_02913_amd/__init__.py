"""SFC (Symbolic Fourier Convolution) 3x3 int8 convolution for MI355X (gfx950).

The compute path is a C-ABI shared library of hand-written HIP kernels
(``csrc/``, declared in ``include/sfc.h``); :mod:`.binding` marshals arguments
to it and nothing else.  There is no CPU fallback: calling into the library
when it has not been built raises.
"""
from . import synth  # noqa: F401

__all__ = ["synth", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib

        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
