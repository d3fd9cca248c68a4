"""MI355X-native double-sampled low-precision SGD (ZipML hot path).

``paper_1611_05402_amd.zipml`` is the thin ctypes binding of the C-ABI library
``libzipml.so`` (hand-written HIP kernels for gfx950); ``paper_1611_05402_amd.synth``
generates the seeded synthetic workloads.  Nothing is loaded at import time; the
binding raises if the library has not been built.
"""
__all__ = ["zipml", "synth"]
