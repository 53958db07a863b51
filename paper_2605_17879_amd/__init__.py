"""MI355X-native hot path of Guard's online straggler detection.

The work is done by hand-written HIP kernels for gfx950 behind the C ABI of
``include/guard.h``; this package only loads that library and marshals
arguments (``guard.py``).  There is no CPU fallback: importing succeeds without
the library, calling anything raises.
"""
from .guard import (  # noqa: F401
    Config,
    Detector,
    GuardError,
    library_path,
    load_library,
)
