"""MGLU forward (Mixture-of-Element-wise-Gating projection) for MI355X / gfx950.

The work is done by hand-written HIP kernels behind a C ABI (`libmglu.so`,
declared in include/mglu.h); `paper_2506_23225_amd.api` is the thin binding.
"""
__version__ = "0.1.0"
