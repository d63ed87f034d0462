"""MI355X (gfx950) batch-1 MoE decode with cache-conditional routing: Python binding of libmoe_cache.

Importing the package loads the HIP library; there is no CPU fallback.  If the library has not been
built the import raises, naming the build command.
"""
from .binding import *  # noqa: F401,F403
from .binding import LIB_PATH, lib  # noqa: F401
from .runtime import ExpertStore, MoEDecoder  # noqa: F401
