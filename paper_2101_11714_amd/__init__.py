"""TT-EmbeddingBag forward/backward for MI355X (gfx950).

The package holds the HIP kernels (``csrc/``), the ctypes binding to the C-ABI
library (``binding``) and the seeded synthetic workload generators
(``workloads``).  Importing the package loads nothing native; the binding is
loaded on first use and raises if the HIP library has not been built.
"""

__all__ = ["binding", "workloads"]
