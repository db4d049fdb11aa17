"""MI355X (gfx950) u8 x s8 -> s32 GEMM: thin ctypes binding over the C-ABI HIP library."""
from .binding import *  # noqa: F401,F403
from .binding import EXPORTS, LIB_PATH, NgemmError  # noqa: F401
