"""MI355X-native decode / chunked-prefill engine (libld) -- Python binding.

The package is a thin ctypes layer over the C-ABI library built from csrc/ (see
include/ld.h, include/ld_kernels.h).  Every step of the path runs in the HIP kernels;
Python only marshals arguments.  Importing the binding fails loudly if the library
has not been built.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
