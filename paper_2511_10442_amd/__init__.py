"""MI355X-native binned exact k-nearest-neighbour graph build (FastGraph, Section 3).

The package holds the HIP kernels + C-ABI library (``csrc/``), a thin ctypes
binding with the same names (``binding``) and the seeded input generators
(``workloads``).  Nothing here falls back to a CPU implementation: if the HIP
library is missing the binding raises.
"""
__all__ = ["binding", "workloads"]
