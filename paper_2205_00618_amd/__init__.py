"""Dense contraction kernels (fp32 GEMM, NHWC direct convolution, s8->s32 GEMM) for gfx950.

The compute lives in the HIP shared library built from ``csrc/``; ``binding`` marshals
arguments to its C ABI and ``workloads`` draws the seeded synthetic inputs.  Nothing is
loaded at import time: ``binding.load()`` opens the library on first use and raises if it
has not been built.
"""

__all__ = ["binding", "workloads", "build"]
