"""MI355X-native HiKonv: packed low-bitwidth convolution behind a C ABI (libhikonv.so)."""
from .binding import *  # noqa: F401,F403
from .binding import Plan, HikonvError, lib, LIB_PATH, SIGNATURES  # noqa: F401
