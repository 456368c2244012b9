"""MI355X-native reduced-precision NMT training step: HIP kernels behind a C ABI (libnmt.so), a
ctypes binding with the same names, and the device-memory plumbing around them."""
from .binding import *  # noqa: F401,F403
from .binding import NmtError, load, exported_symbols, LIB_PATH  # noqa: F401
