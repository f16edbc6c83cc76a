"""Adaptive Block-Sparse Attention (ASA) for MI355X (gfx950).

The package holds the HIP kernels and their C-ABI library (``csrc/``), a thin
ctypes binding with the same entry-point names (``binding``), and the seeded
synthetic input generators (``synth``).  Importing the package does not load
the native library; ``binding.load()`` does, and raises if it is missing.
"""

__all__ = ["binding", "synth"]
