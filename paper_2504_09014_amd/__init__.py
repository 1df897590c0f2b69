"""MI355X-native collective data-movement kernels for N ranks emulated inside one GPU.

Thin ctypes binding over libmsx.so (the C ABI in include/msx.h).  Argument marshalling
only: every step of every collective runs in the HIP kernels.  There is no CPU fallback;
if the library is not built or the call fails, an exception is raised.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
