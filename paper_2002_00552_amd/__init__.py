"""MI355X-native forward convolution by the Decomposable Winograd Method.

The product is libdwm.so (HIP kernels + host planner behind a C ABI, see include/dwm.h);
this package is its thin ctypes binding.  PyTorch is only used by callers for device
memory and streams.
"""
from .binding import *  # noqa: F401,F403
from .binding import DwmError, EXPORTS, LIB_PATH, lib  # noqa: F401
