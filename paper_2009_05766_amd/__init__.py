"""MI355X-native NetMax iteration: thin Python binding of libnetmax.so (HIP kernels, C ABI)."""
from .binding import *  # noqa: F401,F403
from .binding import NetMax, NetmaxError, load, EXPORTS, LIB_PATH  # noqa: F401
