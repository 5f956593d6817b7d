"""MI355X-native hot path of FreeScale's prioritized embedding updates (one GPU, one shard).

The product is ``libfreescale_hip.so`` (hand-written HIP kernels for gfx950 behind the C ABI of
``include/freescale.h``); this package only binds it for Python.
"""
from .binding import *  # noqa: F401,F403
from .binding import Context, FreeScaleError, fs_step_args, load_library, declared_symbols, LIB_PATH  # noqa: F401
