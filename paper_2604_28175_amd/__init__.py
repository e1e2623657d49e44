"""MI355X-native hot path of a dual-priority inference server: hand-written gfx950 kernels
behind a small C ABI (include/strait.h), with a thin ctypes binding of the same names."""
from .binding import *  # noqa: F401,F403
from . import binding  # noqa: F401
