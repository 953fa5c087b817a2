"""Pooled hashed-embedding lookup and sparse row-wise Adagrad on MI355X (gfx950).

The package is a thin ctypes binding over a C-ABI library of hand-written HIP
kernels (``csrc/``), plus the seeded synthetic workload generators.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads"]
