"""MI355X-native preemptive daemon-kernel collectives (the hot path of arXiv 2303.06324).

The product is the HIP library `libdfx.so` (C ABI in include/dfx.h); this package is the thin
ctypes binding over it.  Importing it requires the built library: there is no CPU path.
"""
from .binding import *  # noqa: F401,F403
from .binding import Context, Config, DfxError, config_default, strerror, copy_calibrate, LIB_PATH  # noqa: F401
