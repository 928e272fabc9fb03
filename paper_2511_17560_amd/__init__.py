"""MI355X-native implementation of the per-layer A^3 KV-cache fusion path (arXiv 2511.17560).

``api``   ctypes binding of liba3.so (HIP kernels behind a C ABI, see include/a3.h)
``layer`` the call sequence of one layer on preallocated buffers
``build`` compiles liba3.so with hipcc for gfx950

Importing the package does not load the library; ``api.lib()`` does, and raises if it is missing.
"""
__all__ = ["api", "layer", "build"]
