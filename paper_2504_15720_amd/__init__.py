"""MI355X-native unified-KV decode path: C-ABI library (csrc/) and its ctypes binding.

The HIP library is the product; this package only loads it.  Nothing here computes
attention on the CPU: if libukv.so is missing the calls raise.
"""
from .binding import *  # noqa: F401,F403
from .binding import BatchDesc, UkvError, lib, LIB_PATH, EXPORTS  # noqa: F401
