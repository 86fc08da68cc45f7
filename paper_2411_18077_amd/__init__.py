"""MiniKV decode-step attention over a 2-bit, adaptively evicted KV cache for AMD MI355X (gfx950).

The product is the C library `libminikv.so` (hand-written HIP, C ABI in include/minikv.h); this package
holds its sources (csrc/), the in-tree build (build.py), a ctypes binding with the same entry-point names
(api.py) and seeded synthetic workloads (workloads.py).
"""
from . import api, workloads  # noqa: F401
