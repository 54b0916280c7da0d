"""MI355X-native bit-serial GEMM / convolution on 1-4 bit operands (arXiv 2207.08820, Section V).

The compute lives in hand-written HIP kernels behind a C ABI (``include/dlrt.h``); ``binding``
is a thin ctypes layer over it and ``inputs`` holds the seeded synthetic workloads.  Importing
the package does not load the GPU library; the first call into ``binding`` does, and raises if
the library has not been built.
"""

__all__ = ["binding", "inputs"]
