"""MI355X-native implementation of ARL-Tangram's action-level elastic scheduling step.

``tg`` is the ctypes binding of the C-ABI HIP library (include/tg.h); ``build`` compiles it.
"""
from . import build, tg  # noqa: F401
