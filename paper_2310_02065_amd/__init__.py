"""MI355X-native V:N:M sparse x dense product (the Spatha-style SpMM hot path).

The compute lives in a C-ABI shared library built from csrc/ (HIP, gfx950); `binding` is the
thin ctypes layer over it.  Importing the package does not load the library; `binding.lib()`
does, and raises if it has not been built.
"""
__all__ = ["inputs", "binding"]
