"""MI355X-native decoder-layer kernels (gfx950 HIP) behind the C ABI of include/tessera.h.

This package is a thin ctypes binding: argument marshalling only.  Every step of
the layer runs in the hand-written HIP kernels of libtessera.so; there is no CPU
or PyTorch fallback, and importing `binding` fails loudly when the library has
not been built (python -m paper_2604_10180_amd.build).
"""
from .binding import *  # noqa: F401,F403
