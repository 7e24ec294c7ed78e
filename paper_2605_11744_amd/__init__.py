"""Segment-level causal attention for AMD MI355X (gfx950): Python binding of libsegattn.

The product is the HIP library behind include/segattn.h; this package only marshals
arguments for it (see binding.py).  Importing the package does not load the library;
the first call does, and fails loudly if it has not been built."""
from .binding import *  # noqa: F401,F403
from .binding import EXPORTS, LIB_PATH, SegattnError, lib, make_config, segattn_config  # noqa: F401
