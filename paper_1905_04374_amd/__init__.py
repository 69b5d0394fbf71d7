"""MI355X-native multi-Bulyan gradient aggregation (arxiv 1905.04374).

The work is done by hand-written HIP kernels in libmbulyan.so (C ABI in
include/mbulyan.h); this package is the thin Python binding.  Importing it
fails if the library has not been built: there is no fallback path.
"""
from .binding import *  # noqa: F401,F403
from .binding import EXPORTS, LIB_PATH, MBulyanError, lib  # noqa: F401
