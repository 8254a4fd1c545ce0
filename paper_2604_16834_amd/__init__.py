"""MI355X-native RNS-CKKS batched-convolution hot path (hand-written HIP for gfx950 behind a C
boundary, ``include/ckks.h``).  This package is only the thin binding; see ``binding.py``."""
from .binding import *  # noqa: F401,F403
from .binding import Context, Key, CkksError, from_host, to_host, empty, EXPORTS, LIB_PATH  # noqa: F401
