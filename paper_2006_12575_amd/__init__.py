"""MI355X (gfx950) compute library for the per-device hot path of LAMP's large 3D U-Net
(arXiv 2006.12575): hand-written HIP kernels behind a C ABI (include/lamp.h) and this thin
ctypes binding.  There is no CPU fallback: the functions raise if liblamp.so is not built."""
from .binding import *  # noqa: F401,F403
from .binding import EXPORTS, LIB_PATH, LampError, lib  # noqa: F401
