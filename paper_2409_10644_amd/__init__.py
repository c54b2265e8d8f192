"""MI355X-native verification hot path of multi-candidate speculative decoding (arXiv 2409.10644).

Thin ctypes binding over libmcsd.so (hand-written HIP for gfx950).  Functions have the names of the C ABI
declared in include/mcsd.h and only marshal arguments; PyTorch is used for device memory and streams.
There is no CPU fallback: importing `binding` raises if the library has not been built.
"""

__all__ = ["binding"]
