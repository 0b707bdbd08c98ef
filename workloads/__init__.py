"""Seeded synthetic inputs for the token-routed any-precision linear layer.

This package only *draws inputs* (weights, activations, router parameters) with the
shapes and value structure of Llama-style linear layers.  It holds none of the
method's arithmetic (no quantiser, no slice packing, no routing decision, no GEMM
of the layer itself): both the CPU oracle's tests and the GPU tests/bench take their
inputs from here so that the two sides see bit-identical arrays.
"""
from .generate import (  # noqa: F401
    CONFIGS,
    LinearSpec,
    WorkloadConfig,
    f32_to_bf16_bits,
    make_case,
    make_mlp_router,
    make_router,
    make_tokens,
    make_weight,
)
