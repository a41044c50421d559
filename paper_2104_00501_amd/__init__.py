"""MI355X-native minibatch step of sparse-parameter SGD for the NuPS workloads.

The package holds the HIP kernels and their C-ABI (``csrc/``), a thin ctypes
binding with the same names (``binding``) and the seeded synthetic input
generators (``workloads``).  Importing the package loads nothing native; the
shared library is opened on first use of ``binding`` and its absence is an
error, never a fallback.
"""

__all__ = ["binding", "workloads"]
