"""MI355X-native exact attention forward (the hot path of FastAttention, arXiv 2410.16663).

``fa_fwd`` and friends live in :mod:`paper_2410_16663_amd.binding` (a ctypes view of the
C-ABI library built from ``csrc/``); :mod:`paper_2410_16663_amd.inputs` holds the seeded
synthetic workloads.  Importing the package loads neither torch nor the HIP library.
"""
__all__ = ["binding", "inputs", "build"]
