"""MI355X-native FP8 hot path of FOG-style training: per-tensor casts, scaled FP8 GEMMs, FP8 attention.

`fog` is the thin binding over the C-ABI library (HIP kernels for gfx950);
`synth` holds the seeded synthetic-input generators (no arithmetic of the method).
Importing the package loads nothing native; the first call into `fog` does, and
fails loudly when the library has not been built.
"""
from . import synth  # noqa: F401

__all__ = ["synth", "fog"]


def __getattr__(name):
    if name == "fog":
        import importlib
        return importlib.import_module(__name__ + ".fog")
    raise AttributeError(name)
