"""MI355X-native hybrid-sparse (block AND N:M) GEMM path of CRISP (arXiv 2311.14272).

`synth` holds the seeded synthetic workloads; `crisp` is the thin ctypes binding of
libcrisp.so (HIP kernels for gfx950 behind a C ABI).  Importing the package does not load
the library; the first call into `crisp` does, and fails loudly if it has not been built.
"""
