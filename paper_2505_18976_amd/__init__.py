"""GraSS / FactGraSS per-sample gradient compression for AMD MI355X (gfx950).

The product is libgrass.so (hand-written HIP kernels behind the C ABI declared
in include/grass.h).  This package only marshals arguments: see binding.py.
"""
from .binding import *  # noqa: F401,F403
from .binding import load_library, GrassError, SIGNATURES, LIB_PATH  # noqa: F401
