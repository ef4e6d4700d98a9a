"""Seeded synthetic workload generators shared by the tests, the bench and the oracle checks.

This package holds input preparation only: random gate weights, random expert
weights and their min/max group quantization into (codes, scale, zero), and
the hidden-state streams.  It contains none of the decode path's arithmetic
(no gating, no dequantization, no FFN, no cache logic) and imports neither the
HIP binding nor the CPU oracle.
"""
from .generate import (  # noqa: F401
    CONFIGS,
    MoEShape,
    stream_seed,
    gate_weight,
    rms_gamma,
    expert_matrix_shape,
    expert_matrix,
    quantize_minmax,
    quantize_meta8,
    run_length,
    quantized_expert,
    hidden_iid,
    hidden_ar1,
    layer_formats,
)
