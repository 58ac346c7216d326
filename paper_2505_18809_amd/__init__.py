"""VORTA routed attention for AMD MI355X (gfx950).

The product is libvorta.so (csrc/, C ABI in include/vorta.h); this package is its thin
ctypes binding.  Importing it does not load the library; the first call does, and raises
if the library cannot be loaded -- there is no CPU or PyTorch fallback.
"""
from .binding import *  # noqa: F401,F403
from .binding import Plan, VortaError, load_library, plan_for, LIB_PATH, SYMBOLS  # noqa: F401
