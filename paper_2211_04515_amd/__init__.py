"""MI355X (gfx950) activation compression for pipeline-stage boundaries (QuantPipe's PDA path).

Thin ctypes binding over libquantpipe.so; every step of the path runs in the HIP kernels.
Importing this package loads the library and raises if it has not been built: there is no
CPU fallback.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
