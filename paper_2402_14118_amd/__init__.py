"""MI355X-native Masked Matrix Multiplication (C = M(X) x N(Y)).

The product is the HIP library `libmmm_hip.so` behind the C ABI of
include/mmm.h; this package is its thin Python binding plus a small helper that
owns the device buffers of one problem.
"""
from .binding import *          # noqa: F401,F403
from .binding import MaskA, MaskB, MmmError, lib, LIB_PATH, EXPORTS   # noqa: F401
from .engine import MaskedMatmul                                     # noqa: F401
