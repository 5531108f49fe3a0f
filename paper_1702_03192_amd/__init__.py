"""MI355X-native NT-operation path of MTNN: direct NT GEMM, transpose + NN GEMM (TNN) and a
boosted-tree selector between them, as hand-written HIP kernels behind a C-ABI library.

The HIP library is loaded on first use (see ``binding``); importing the package alone touches
neither the GPU nor the library, so the seeded input generators in ``inputs`` can be used anywhere.
"""
__all__ = ["inputs", "binding"]
