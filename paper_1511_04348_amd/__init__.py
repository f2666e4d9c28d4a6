"""tgemm: tiled in-core / out-of-core GEMM and MLP training passes for one MI355X (gfx950).

The compute path is a C-ABI shared library of hand-written HIP kernels
(``csrc/``, declared in ``include/tgemm.h``); ``binding`` is the thin ctypes
layer over it.  ``inputs`` holds the seeded synthetic input generators and
none of the method's arithmetic.  Importing this package does not load the
library; the first call through ``binding`` does, and fails loudly if the
library has not been built.
"""
__all__ = ["binding", "inputs"]
