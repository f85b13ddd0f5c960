"""txops: ATen-semantics tensor operators as hand-written HIP kernels for gfx950 (MI355X).

The compute lives in csrc/ behind a C ABI (include/txops.h); `binding` is the
thin ctypes layer with the same entry-point names; `inputs` holds the seeded
synthetic input generators.  Importing the package does not load the native
library; the first call into `binding` does, and raises if it is missing.
"""
__all__ = ["binding", "inputs"]
