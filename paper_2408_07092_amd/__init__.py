"""Double Sparsity decode attention for MI355X (gfx950): Python face of libdsattn.

The package is a thin binding over the C-ABI library built from ``csrc/``; see
``include/ds_attn.h`` for the contract of every call.
"""
from .binding import *  # noqa: F401,F403
from .binding import DsError, DsShape, lib, shape, strerror  # noqa: F401
