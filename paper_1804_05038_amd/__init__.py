"""MI355X-native hot path of 8-bit GRU-NMT decoding ("Pieces of Eight", Quinn & Ballesteros).

The product is libq8nmt.so, a C-ABI library of hand-written gfx950 kernels declared in
include/q8nmt.h.  This package is a thin ctypes binding with the same entry-point
names; torch supplies device memory and the stream, nothing else.  There is no CPU
fallback: importing `binding` fails loudly if the library has not been built.
"""
from .binding import *  # noqa: F401,F403
