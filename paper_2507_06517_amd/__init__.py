"""MI355X-native prefill-time KV-cache reduction pass of SpindleKV.

Two device entry points behind a C-ABI library (``include/spindle.h``):
attention-weight eviction for deep layers and similarity-codebook replacement
for shallow layers.  This package holds the HIP sources (``csrc/``), the thin
``ctypes`` binding (``binding``) and the seeded synthetic input generators
(``workloads``).  Importing the package loads nothing native; the binding
loads the shared library on first use and raises if it is missing.
"""

__all__ = ["binding", "workloads"]
