"""CPU oracle for the fused RMSNorm -> MatMul operator family (test infrastructure).

This package is the slow, plain, fp64 definition of what the HIP library
computes.  It exists only to check that library: the tests, the smoke entry
and the benchmark's ``cpu_baseline`` leg are its only callers.  It shares no
code with the HIP path and never imports it.
"""
from .rmsnorm_family import (  # noqa: F401
    rms_norm,
    rmsnorm_matmul,
    rmsnorm_gated_mlp,
    rmsnorm_glu,
    swiglu,
    softmax_matmul,
    gqa_decode_attention,
    silu,
)
