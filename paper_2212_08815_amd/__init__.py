"""MI355X-native sparse-filter / sparse-input 2-D convolution (FSCNN hot path).

`paper_2212_08815_amd.fscnn` is the thin ctypes binding of the C-ABI library
declared in include/fscnn.h; `paper_2212_08815_amd.inputs` draws the seeded
synthetic workloads.  Importing the package loads nothing; the binding loads
libfscnn.so on first use and raises if it has not been built.
"""
__all__ = ["fscnn", "inputs"]
