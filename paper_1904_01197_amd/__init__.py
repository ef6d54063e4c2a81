"""libndq: dithered (DQSG) and nested dithered (NDQSG) gradient quantization on MI355X.

The compute path is the C-ABI shared library ``libndq.so`` (hand-written HIP
kernels for gfx950, declared in ``include/ndq.h``); this package is a thin
ctypes binding over it (``paper_1904_01197_amd.ndq``) plus seeded synthetic
workloads (``paper_1904_01197_amd.workloads``).  The library is loaded on
first use and there is no CPU fallback: without it every call raises.
"""
__all__ = ["ndq", "workloads"]
