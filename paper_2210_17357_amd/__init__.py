"""MI355X-native L-GreCo hot path: per-layer compression-error profiler, the layer x
error-bin dynamic program and the per-layer compressors, as HIP kernels for gfx950 behind
a C-ABI library (liblgreco.so).  This package holds the kernels' sources (csrc/), the ctypes
binding (binding.py) and the seeded synthetic workloads (workloads.py)."""
from . import workloads  # noqa: F401

__all__ = ["workloads", "binding"]
