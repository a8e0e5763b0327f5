"""MI355X-native TSR-Adam per-matrix optimizer path: thin Python binding over libtsr.so.

Every step of the path runs in the HIP kernels of the C-ABI library declared in
include/tsr.h; this package only marshals arguments (tensor pointers, sizes, stream).
There is no CPU or PyTorch fallback: importing `binding` fails if the library is missing.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
