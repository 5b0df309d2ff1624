"""MI355X-native convolution-layer operators and single-GPU bi-graph executor.

`binding` mirrors the C ABI of include/purine.h one to one; `layers` builds the synthetic
workload graphs on top of it. The HIP library is the only compute path: importing this package
fails if libpurine_conv.so has not been built.
"""
from .binding import *  # noqa: F401,F403
from . import binding  # noqa: F401
