"""Block-sparse cached-activation convolution and sparse-query attention for MI355X.

The compute lives in a C-ABI shared library of hand-written HIP kernels
(``csrc/``, declared in ``include/sige.h``); :mod:`.api` is the thin ctypes
binding with the same entry-point names, :mod:`.inputs` the seeded synthetic
workloads.  Importing the package does not load the library; the first call
into :mod:`.api` does, and fails loudly when it has not been built.
"""
__all__ = ["api", "inputs"]
