"""DynSplit-KV hot path for AMD MI355X: HIP kernels behind a C ABI (libdsk.so) and a thin
ctypes binding.  Importing the package loads the library; there is no fallback path."""
from .binding import *  # noqa: F401,F403
from . import binding  # noqa: F401
