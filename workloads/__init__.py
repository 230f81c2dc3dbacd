"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests and bench.

This package draws random numbers and converts storage formats; it contains none of the
decoder-layer arithmetic, none of the oracle and none of the GPU library.
"""
from .gen import (  # noqa: F401
    CONFIGS,
    DecoderShape,
    bf16_bits_from_f32,
    f32_from_bf16_bits,
    layer_weights_bits,
    hidden_bits,
    kv_prefill_bits,
    lognormal_lengths,
    uniform_lengths,
    TENSOR_ORDER,
    tensor_shapes,
)
