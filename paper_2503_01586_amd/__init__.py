"""EliteKV decode hot path for AMD MI355X: a ctypes binding over libelitekv.so (HIP, gfx950).

The package holds the kernels (csrc/), the build script and the binding; nothing else.  Importing
it requires the built library; there is no CPU fallback.
"""
from .binding import *  # noqa: F401,F403
from .binding import (EXPORTS, LIB_PATH, EliteKVError, elitekv_dims, make_dims, raw, torch_dtype)  # noqa: F401
