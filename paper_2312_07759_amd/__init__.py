"""MI355X-native implicit differentiable soft k-means (IDKM hot path).

`binding` wraps the C ABI of libidkm.so (include/idkm.h); `workloads` draws the
seeded synthetic inputs; `build` compiles the library in-tree with hipcc.
"""
from . import workloads  # noqa: F401  (numpy only)

__all__ = ["workloads", "binding", "build"]
