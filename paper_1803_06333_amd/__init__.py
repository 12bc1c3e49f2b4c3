"""MI355X-native local solver of Snap ML (arXiv 1803.06333, Section 3.1-3.2): asynchronous
stochastic coordinate descent for GLMs as hand-written HIP kernels behind a C ABI
(include/snap.h).  This package holds the HIP sources (csrc/), their build step and a ctypes
binding; there is no CPU fallback."""
from .binding import (Solver, SnapError, load_library, make_matrix, perm_key, block_order, stream_probe, EXPORTS, CSR, CSC, DENSE_ROWMAJOR,
                      DENSE_COLMAJOR, RIDGE, LOGISTIC, HINGE, FORM_AUTO, PRIMAL, DUAL)

__all__ = ["Solver", "SnapError", "load_library", "make_matrix", "perm_key", "block_order", "stream_probe", "EXPORTS"]
