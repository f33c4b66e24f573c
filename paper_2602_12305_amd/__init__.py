"""MI355X-native fused dense contraction  C = act(A.B + bias).

The package holds the HIP kernels and C-ABI library (``csrc/``), a thin ctypes
binding with the same entry-point names (``binding``), and the profiler-driven
variant sweep and tree search (``sweep``, ``search``).  The seeded synthetic input
generators live outside the package, in the top-level ``inputs`` package.

Importing the package loads nothing native; the shared library is opened on
the first call through ``binding`` and a missing library is a hard error.
"""

__all__ = ["binding"]
