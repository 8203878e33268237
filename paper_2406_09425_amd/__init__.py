"""MI355X-native stage computation under SGPRS: thin Python binding of libsgprs.

Every function here only marshals arguments into the C ABI declared in
include/sgprs.h; all computation runs in the library's HIP kernels.  There is
no CPU fallback: if libsgprs.so is missing or a call fails, an exception is
raised.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
