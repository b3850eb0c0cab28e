"""MI355X-native tree-attention decode (DeFT-Flatten hot path).

The package holds the HIP/C++ sources of ``libdeft.so`` (``csrc/``), the thin
ctypes binding over its C ABI (``binding``) and the seeded synthetic workload
generators (``workloads``).  Importing the package loads nothing native; the
binding loads the shared library on first use and raises if it is missing.
"""

__all__ = ["binding", "workloads"]
