"""Seeded synthetic inputs (model shapes, weights, prompts) shared by the oracle and the HIP path.

This package holds no arithmetic of the decoding method itself: it only names the
workload shapes and fills arrays from seeded random streams.
"""
from .synth import (  # noqa: F401
    ModelConfig,
    Workload,
    CONFIGS,
    get_workload,
    make_weights,
    make_tensor,
    make_prompt,
    WEIGHT_NAMES_PER_LAYER,
    shrink,
    f32_to_bf16_bits,
    iter_tensor_keys,
)
