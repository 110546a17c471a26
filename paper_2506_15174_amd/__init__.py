"""MI355X (gfx950) sparse-times-dense product, C = A x B, behind a small C ABI.

The product path is the shared library built from ``csrc/`` (host inspector in
C++, executor in hand-written HIP); this package only marshals arguments.
"""
from .binding import (Plan, SpmmError, plan_create, load, status_string, LIB_PATH,
                      SPMM_OK, SPMM_ERR_INVALID_ARG, SPMM_ERR_INVALID_CSR, SPMM_ERR_ALLOC,
                      SPMM_ERR_HIP, SPMM_ERR_UNSUPPORTED,
                      ARRAY_HDR, ARRAY_STREAM, ARRAY_WINS, ARRAY_ITEMS, ARRAY_ROWMAP, ARRAY_CROSS, EXPORTS)

__all__ = ["Plan", "SpmmError", "plan_create", "load", "status_string", "LIB_PATH", "EXPORTS"]
