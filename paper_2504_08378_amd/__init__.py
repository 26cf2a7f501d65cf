"""MI355X-native active-weight decode path (ActiveFlow, arXiv 2504.08378).

`paper_2504_08378_amd.binding` is a thin ctypes layer over libactiveflow.so (hand-written
HIP for gfx950, C ABI in include/activeflow.h).  Importing this package does not load the
library; `binding.lib()` does, and raises if it has not been built.
"""
__all__ = ["binding", "build", "model"]
