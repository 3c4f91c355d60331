"""MI355X-native data-movement primitives and partitioned layers of
arXiv 2006.03108, as a C-ABI HIP library (libdistdl.so) with a thin ctypes
binding.  Importing this package loads the library and fails loudly if it
has not been built (python paper_2006_03108_amd/build.py)."""
from .binding import *  # noqa: F401,F403
from .binding import lib, DistdlError  # noqa: F401
