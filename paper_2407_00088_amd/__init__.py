"""MI355X-native LUT-based mixed-precision GEMV/GEMM (T-MAC hot path), gfx950 only.

The product is the C-ABI shared library ``libtmac_hip.so`` declared in ``include/tmac.h``;
this package is its thin Python binding.
"""
from .binding import *  # noqa: F401,F403
from .binding import lib, LIB_PATH, EXPORTS, TmacError  # noqa: F401
from .runner import LinearLUT  # noqa: F401
