"""MI355X-native SALAD attention forward: HIP kernels behind a C ABI (include/salad.h) and a thin
ctypes binding.  `workloads` holds the seeded synthetic inputs; `binding` the entry points."""
from . import workloads  # noqa: F401

__all__ = ["workloads", "binding"]
