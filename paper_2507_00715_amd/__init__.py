"""EARN register-token attention hot path for one MI355X (gfx950).

`workloads` draws seeded synthetic inputs; `binding` is the thin ctypes layer over
libearn.so (hand-written HIP kernels behind a C ABI).  Importing the package does
not load the library; `binding.lib()` does, and raises if it has not been built.
"""
__all__ = ["workloads", "binding", "build", "pipeline"]
