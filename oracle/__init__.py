"""CPU oracle for the FP8 hot path (casts, scaled GEMMs, FP8 attention).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, float64 statement of
what the GPU library must compute.  It is imported by the tests, by the smoke
check and by the benchmark's CPU-baseline leg, and by nothing else; the product
path never falls back to it.  It shares no code with the HIP kernels and never
imports the GPU package.

Every function cites the passage of the paper (section / equation / appendix)
that defines what it computes.  Pins for each function live in the CPU test
suite; none is "parity unpinned".
"""
from . import bf16, fp8, scaling, gemm, attention, kurtosis, qknorm, xielu, gelu, postnorm  # noqa: F401
