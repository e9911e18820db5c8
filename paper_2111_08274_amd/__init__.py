"""HADFL aggregation-cycle hot path for MI355X (gfx950).

``paper_2111_08274_amd.hadfl`` is the thin binding over the C-ABI library
``libhadfl.so`` (hand-written HIP kernels); ``paper_2111_08274_amd.synth`` holds
the seeded synthetic-input generators.  Importing the package loads neither.
"""
__all__ = ["hadfl", "synth"]
