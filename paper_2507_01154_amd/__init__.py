"""MI355X-native per-layer DP weight-gradient path (FlashDP, Algorithm 1): a C-ABI HIP library
(csrc/, include/flashdp.h) and its thin ctypes binding."""
from .binding import *  # noqa: F401,F403
from .binding import lib, FlashDPError  # noqa: F401
