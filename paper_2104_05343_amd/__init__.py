"""MI355X-native per-device hot path of the 2D (SUMMA) transformer scheme of arXiv 2104.05343.

The product is ``liboptimus.so`` (hand-written HIP for gfx950 behind a C ABI, see include/optimus.h).
This package only marshals arguments: every step of the path runs in the library's kernels.  There is
no CPU fallback: importing ``binding`` fails loudly when the library has not been built.
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
