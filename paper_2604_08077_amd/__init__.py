"""AdaS-Attn (Adaptive Cube-Selective Attention) for MI355X / gfx950.

The compute path is a C-ABI HIP library (``csrc/`` -> ``libadaspark.so``);
``binding`` marshals arguments into it and ``synth`` generates the seeded
synthetic workloads.  Importing the package does not load the library; any call
that needs it raises if it has not been built.
"""
from . import synth  # noqa: F401

__all__ = ["synth", "binding", "build"]


def __getattr__(name):
    if name in ("binding", "build"):
        import importlib

        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
