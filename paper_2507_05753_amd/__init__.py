"""Jigsaw-partitioned linear layer forward (Y = X W^T + b, 1/2/4-way) for MI355X.

``inputs``  - seeded synthetic input generators (no method arithmetic).
``binding`` - ctypes binding of the C-ABI library ``libjigsaw.so`` (HIP kernels).

Importing the package loads nothing heavy; ``binding`` raises at import time if
the HIP library has not been built (there is no CPU fallback).
"""

__all__ = ["inputs", "binding"]
