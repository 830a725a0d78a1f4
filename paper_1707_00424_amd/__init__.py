"""Parle replica-coupled training step for MI355X (gfx950).

The product path is the C-ABI library built from ``csrc/`` and the thin ctypes
binding in :mod:`paper_1707_00424_amd.binding`.  This package file imports
nothing heavy so that :mod:`paper_1707_00424_amd.synth` (seeded input
generators, numpy only) can be used without the HIP library.
"""

__all__ = ["synth", "binding", "build"]
