"""Fier decode hot path for one MI355X: thin Python binding over the C-ABI library libfier.so.

``synth`` (seeded inputs) is importable without the library; everything in ``binding`` needs it and
fails loudly when it is missing -- there is no CPU fallback.
"""
__all__ = ["binding", "synth", "build"]
