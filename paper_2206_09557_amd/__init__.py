"""MI355X-native LUT-GEMM: BCQ weight-only quantised GEMV / small-batch GEMM by table
lookup.  The work is done by liblutgemm.so (hand-written HIP for gfx950, C ABI declared
in include/lutgemm.h); this package is its ctypes binding plus seeded input generators."""
from .lutgemm import *  # noqa: F401,F403
from .lutgemm import EXPORTS, LIB_PATH, LutGemmError, lib  # noqa: F401
