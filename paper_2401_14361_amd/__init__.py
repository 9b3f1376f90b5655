"""MI355X-native decode hot path of a sparsity-aware MoE expert cache.

The product is the HIP library ``libmoei.so`` (C ABI in ``include/moei.h``);
``binding`` is the thin ctypes layer over it.  Nothing here computes on the CPU.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
