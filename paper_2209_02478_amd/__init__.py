"""MI355X-native checkpointed training step with an input-aware planner (libmimose).

Thin ctypes binding over the C ABI declared in include/mimose.h: argument marshalling
only, every step of the path runs in the library's HIP kernels.  The shared library
must have been built (paper_2209_02478_amd/build.py); loading fails loudly otherwise.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
