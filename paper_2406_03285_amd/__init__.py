"""Per-GPU rehearsal buffer for MI355X (gfx950): C-ABI HIP library plus a ctypes binding.

Importing this package loads paper_2406_03285_amd/librb.so and fails if it has
not been built (`python paper_2406_03285_amd/build.py`); there is no CPU path.
"""
from .binding import *  # noqa: F401,F403
from .binding import RehearsalBuffer, Pipeline, RbError, EXPORTS, LIB_PATH  # noqa: F401
