"""MI355X-native per-task MAML step over a DLRM-style model (G-Meta's data-parallel hot path).

The product is libgmeta.so (hand-written HIP kernels behind the C ABI of
include/gmeta.h); this package is its thin Python binding.
"""
from .binding import GMeta, GMetaError, load_library, LIB_PATH, EXPORTS

__all__ = ["GMeta", "GMetaError", "load_library", "LIB_PATH", "EXPORTS"]
