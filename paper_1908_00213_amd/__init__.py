"""MI355X-native array kernels for the training-step hot path of a define-by-run framework.

``binding``   ctypes wrappers of the C ABI in ``include/chn.h`` (HIP kernels in ``csrc/``)
``steps``     training steps written as sequences of those calls
``workloads`` seeded synthetic inputs of the benchmark configurations
``build``     compiles ``libchn.so`` in-tree for gfx950

Nothing is loaded at import time; the first call into ``binding`` loads the built library and fails
loudly when it is missing.
"""
__all__ = ["binding", "steps", "workloads", "build"]
