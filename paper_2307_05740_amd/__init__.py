"""Arrow-matrix-decomposition SpMM for one MI355X (gfx950).

``Y = A.X`` is evaluated as ``sum_i P_i^T . B_i . (P_i . X)`` over arrow matrices
``B_i`` by hand-written HIP kernels behind a small C-ABI (``include/arrow.h``).
The Python layer in :mod:`paper_2307_05740_amd.binding` only marshals arguments.
"""
__all__ = ["binding", "synth"]
