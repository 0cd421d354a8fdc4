"""MI355X-native implementation of Flora's hot path (arXiv 2402.03293):
random-projection compression of weight gradients with the projection
regenerated from a seed.  The work is done by hand-written gfx950 kernels
behind a C ABI (include/flora.h); ``flora`` is the ctypes binding,
``workloads`` holds the synthetic benchmark shapes and input recipes."""
from . import flora, workloads  # noqa: F401

__all__ = ["flora", "workloads"]
