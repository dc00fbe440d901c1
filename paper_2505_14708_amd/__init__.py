"""MI355X-native DraftAttention hot path (draft-guided block-sparse 3D attention).

``paper_2505_14708_amd.binding`` is the thin ctypes layer over the C-ABI library
built from ``csrc/``; ``paper_2505_14708_amd.workloads`` makes the seeded synthetic
inputs.  Nothing is loaded at import time: importing the package does not need a GPU
or a built library.
"""
__all__ = ["binding", "workloads", "build"]
