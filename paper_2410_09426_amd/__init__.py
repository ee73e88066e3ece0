"""MI355X-native FlatQuant online path: fused Kronecker transform + INT4 quantization.

The compute lives in a C-ABI shared library of hand-written gfx950 kernels
(``csrc/``); ``binding`` marshals arguments to it and nothing else.  Importing
the package does not load the library; the first call does, and raises if it
has not been built (there is no CPU fallback).
"""
from . import synth  # noqa: F401  (pure numpy input generators)

__all__ = ["synth", "binding", "build"]
