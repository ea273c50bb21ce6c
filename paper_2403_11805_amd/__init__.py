"""Chunk-wise KV-cache scoring, compression and swap-in for LLM context
switching (arXiv 2403.11805) on one MI355X: a C-ABI library of hand-written
gfx950 kernels (csrc/, built into libkvswitch.so) and this thin binding.

`synth` (seeded inputs) imports nothing from the binding; the binding is loaded
on first attribute access so that importing the package never needs the library.
"""
from __future__ import annotations

import importlib

__all__ = ["binding", "build", "synth"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module(f"{__name__}.{name}")
    binding = importlib.import_module(f"{__name__}.binding")
    try:
        return getattr(binding, name)
    except AttributeError:
        raise AttributeError(f"module {__name__!r} has no attribute {name!r}") from None
