"""MI355X-native gated subspace linear layer (hand-written HIP kernels behind a C ABI).

``paper_2605_03109_amd.gsi`` is the ctypes binding of ``libgsi.so`` (loaded on first use; importing
it fails loudly when the library has not been built).  ``paper_2605_03109_amd.workload`` makes the
seeded synthetic operands and needs neither a GPU nor the library.
"""
__all__ = ["workload", "gsi", "build"]
