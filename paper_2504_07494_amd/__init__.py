"""MI355X-native hybrid-cache decode attention (paged KV cache + hidden cache).

The package is a thin binding over a C-ABI shared library of hand-written HIP
kernels for gfx950 (see `binding`), plus the seeded synthetic-input generator
(`workloads`).  Importing the package does not load the library; the first call
into `binding` does, and fails loudly if it has not been built.
"""
__all__ = ["binding", "workloads"]
