"""MI355X-native dynamic-shape contraction library (uKernel patchwork) -- Python binding.

Thin ctypes layer over libftuner.so with the same names as the C ABI in include/ftuner.h.
Argument marshalling only: every step of the path runs inside the library.
"""
from .binding import *  # noqa: F401,F403
