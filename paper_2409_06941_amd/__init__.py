"""MI355X-native bubble harvesting: thin ctypes binding over libfreeride.so (see include/freeride.h).

Argument marshalling only; every step of the path runs inside the library's HIP kernels and host runtime.
The library must have been built (paper_2409_06941_amd/build.py); importing this package fails loudly otherwise.
"""
from .binding import *          # noqa: F401,F403
from .binding import lib, LIB_PATH   # noqa: F401
