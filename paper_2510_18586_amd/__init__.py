"""tokencake_kv for MI355X: paged KV-cache offload / upload behind a C ABI.

The package is a ctypes binding over ``libtokencake_kv.so`` (HIP, gfx950); every step of the
path runs in that library.  There is no CPU fallback: importing works without a GPU, calling
needs one, and a missing library is an ImportError.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
