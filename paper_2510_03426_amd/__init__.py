"""MI355X-native GOOM scans: thin Python binding over libgoom (HIP kernels + C ABI).

The package holds the HIP sources (``csrc/``), the build step (``build.py``) and the
ctypes binding (``binding.py``).  There is no CPU fallback: without the built library
and a gfx950 device every call raises.
"""
from .binding import (  # noqa: F401
    GoomError, Goom, C64, C128, ZERO_NEG_INF, ZERO_FLOOR, LMME_FAST, LMME_EXACT,
    RESET_ALWAYS, RESET_COLINEAR, RESET_NEVER, AFFINE_TIME_INVARIANT, library_path, load_library,
)
