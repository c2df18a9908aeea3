"""MI355X-native real-time pre-ranking scoring path of AIF (arXiv 2511.12934).

``workloads`` makes seeded synthetic inputs; ``binding`` is the thin ctypes
layer over the C-ABI library ``libaif.so`` (HIP kernels for gfx950).  The
library is loaded on first use and a missing build raises: there is no CPU
fallback.
"""
__all__ = ["workloads", "binding"]
