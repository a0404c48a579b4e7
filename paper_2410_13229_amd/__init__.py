"""MI355X-native W8A8 Mamba-mixer path (Quamba, arXiv 2410.13229).

The product is ``libquamba.so`` (hand-written HIP for gfx950 behind the C ABI declared in
``include/quamba.h``).  This package is a thin ctypes binding with the same entry-point
names; it marshals arguments and nothing else.  There is no CPU fallback: every call fails
loudly if the library has not been built (``python -m paper_2410_13229_amd.build``).
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
