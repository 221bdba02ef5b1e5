"""Change-based convolution (CBconv) for MI355X: HIP kernels behind a C ABI
(include/cbconv.h, built into libcbconv.so) and a thin ctypes binding."""
from .binding import *  # noqa: F401,F403
from .binding import Layer, Pool, Network, lib, LIB_PATH, EXPORTS  # noqa: F401
