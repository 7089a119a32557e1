"""Seeded synthetic inputs for the tensor-parallel layer shard.

This package only produces numbers (a counter-based Gaussian generator, the
bf16 storage rounding of inputs, and the named workload shapes).  It contains
none of the layer's arithmetic and is imported by both the CPU oracle's tests
and the GPU path's tests/bench so that both sides see identical inputs.
"""
from .gen import normal, to_bf16_bits, bf16_bits_to_f32, quantize  # noqa: F401
from .configs import LayerConfig, CONFIGS, NEXT_SHAPES, get_config, make_inputs, TENSOR_IDS  # noqa: F401
