"""Seeded synthetic inputs for the DIP / DIP-CA hot path.

This package holds only input recipes and storage-format encoders (random
draws, bf16 rounding of generated weights, int4 packing, the five workload
configurations).  It contains none of the method's arithmetic: no scoring, no
top-k, no GEMV, no cache policy.  Both the CPU oracle's tests and the HIP
path's tests/benchmarks draw their inputs from here so that the two sides see
bit-identical data without sharing any code of the method itself.
"""
from .synth import (  # noqa: F401
    CONFIGS,
    WorkloadConfig,
    ar1_laplace_stream,
    f32_to_bf16_bits,
    gaussian_tokens,
    k_from_ratio,
    layer_weights, layer_weights_split,
    lru_warm_bits,
    pack_int4_g128,
    studentt_tokens,
)
