"""MI355X-native batched hybrid KV-cache restoration (CacheFlow's hot path).

Thin ctypes binding over libcacheflow.so; every step of the path runs in the
library's HIP kernels and host C++.  There is no CPU fallback: importing
`binding` without the built library raises."""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
