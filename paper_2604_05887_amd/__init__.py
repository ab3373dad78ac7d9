"""HybridKV hot path for AMD MI355X: hand-written HIP kernels behind a C ABI (include/hkv.h).

`binding` mirrors the C entry points one to one; `runner` moves synthetic workloads onto the
device.  There is no CPU fallback: without the built libhkv.so every compute call raises.
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
