"""Bipolar-INT arbitrary-precision GEMM for MI355X (gfx950).

The product is the C-ABI library built from ``csrc/`` (see ``include/apmm.h``);
``binding`` marshals arguments to it, ``inputs`` generates seeded synthetic data.
Nothing is loaded at import time; ``binding`` raises if the HIP library is missing.
"""
import importlib

__all__ = ["binding", "inputs"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module(__name__ + "." + name)
    raise AttributeError(name)
