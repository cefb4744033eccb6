"""MI355X-native tensor-contraction operators (GEMM, batched matmul, conv2d) on gfx950 MFMA tiles.

The compute lives in ``csrc/`` (HIP kernels behind a C ABI declared in ``include/tir.h``);
``binding`` is a thin ctypes layer over it.  Importing the package does not load the library.
"""
__all__ = ["binding", "inputs", "buildlib"]
