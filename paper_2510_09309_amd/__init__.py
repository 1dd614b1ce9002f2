"""MaskKV eviction hot path for MI355X (gfx950): C-ABI HIP library plus a thin Python binding.

``synth`` draws the seeded inputs; ``binding`` marshals torch device pointers into the
C-ABI calls of ``libmaskkv.so`` (built from ``csrc/``).  Nothing here computes on the CPU.
"""
from . import synth  # noqa: F401

__all__ = ["synth", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
