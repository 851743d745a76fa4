"""MI355X (gfx950) low-bit GEMM: binary / ternary / ternary-binary matrix multiplication on bit-packed operands.

The work is done by hand-written HIP kernels behind a C ABI (include/lowbit_gemm.h, built into
liblowbit_gemm.so); `binding` marshals torch tensors into that ABI and `synth` draws the seeded benchmark inputs.
Importing the package does not load the library; the first call through `binding` does, and raises if the
library has not been built (there is no CPU fallback).
"""
from . import synth  # noqa: F401

__all__ = ["binding", "synth", "build"]
