"""MI355X-native deeply fused SwiGLU MLP (libdfk) - Python binding of the C ABI.

The package holds the HIP sources (csrc/), the in-tree build (build.py) and
the ctypes binding (binding.py).  Nothing here computes on the CPU.
"""
from .binding import *  # noqa: F401,F403
from .binding import lib, LIB_PATH, dfk_config_t, DfkError, new_workspace  # noqa: F401
