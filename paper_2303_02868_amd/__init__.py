"""apm: page-granular mixed-precision AdamW for MI355X (gfx950).

The product is the C-ABI library (include/apm.h, csrc/); this package is its thin Python binding.
"""
from .binding import *  # noqa: F401,F403
from .binding import lib, LIB_PATH, EXPORTS  # noqa: F401
