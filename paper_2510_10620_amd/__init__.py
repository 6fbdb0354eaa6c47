"""MI355X-native block-attention hot path of Dynamic Context Parallelism (DCP):
a C-ABI library of hand-written gfx950 kernels (csrc/, include/dcp.h) and this thin binding."""
from . import workloads  # noqa: F401
from .api import *  # noqa: F401,F403
