"""psk: position-space sparse x dense kernels for MI355X (gfx950).

The product is the C-ABI library ``libpsk.so`` (see include/psk.h); this package only loads it and
marshals arguments.  Importing the package does not need a GPU; calling an operation does.
"""
from .binding import *  # noqa: F401,F403
from .binding import EXPORTS, LIB_PATH, PskError, lib, status_string, workspace  # noqa: F401
