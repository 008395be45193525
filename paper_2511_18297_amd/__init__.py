"""MI355X-native degree-split SpMM of GROOT (arXiv 2511.18297).

The package is a thin ctypes binding over ``libgroot.so`` (hand-written HIP for
gfx950 behind a C ABI, see ``include/groot.h``).
"""
from .binding import *  # noqa: F401,F403
from .binding import EXPORTS, LIB_PATH, GrootError, Graph, Plan, Parts  # noqa: F401
