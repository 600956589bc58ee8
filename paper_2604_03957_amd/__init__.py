"""BWTA (binary weights, ternary activations) linear hot path for MI355X (gfx950).

``synth`` (seeded inputs) is importable on its own.  Everything else lives in
``binding`` and needs the compiled HIP library ``csrc/libbwta.so``; importing it
fails loudly when the library is missing.  There is no CPU fallback.
"""
import importlib

__all__ = ["synth", "binding"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module("." + name, __name__)
    raise AttributeError(name)
