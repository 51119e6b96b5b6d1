"""GraphVite's GPU training hot path on one MI355X: hand-written gfx950 kernels
behind a C boundary (include/gvhot.h), with this thin ctypes binding on top."""
from .binding import *  # noqa: F401,F403
from .binding import EXPORTS, LIB_PATH, GvError, load  # noqa: F401
