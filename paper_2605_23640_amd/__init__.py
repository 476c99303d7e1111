"""CachePrune's token-granular KV sharing path on AMD MI355X (gfx950):
hand-written HIP kernels behind a C ABI (``include/cacheprune.h``), a ctypes
binding of the same names (``binding``) and a small pool object that strings the
calls together (``pool``).  There is no CPU fallback."""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
from .pool import KVPool, LookupBuffers, LookupResult  # noqa: F401
