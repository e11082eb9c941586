"""MI355X-native LycheeCluster decode hot path: HIP kernels behind a C ABI.

`binding` mirrors the C ABI of liblychee.so (include/lychee.h); `build` compiles it.
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
