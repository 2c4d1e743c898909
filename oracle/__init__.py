"""CPU oracle (test infrastructure) for the block-sparse convolution / sparse-query
attention hot path of Spatially Sparse Inference.

Plain C in double precision (``sige_oracle.c``) reached through ctypes, plus the
few compositions the paper states (Sec. 3.1 identity, Fig. "pipeline" (a) and
(b), Fig. "sige-attention").  Nothing here is imported by the product package
and nothing here imports it.  Only tests, the smoke check and the benchmark's
CPU-baseline leg may use this module.
"""
from .sige_oracle import *  # noqa: F401,F403
