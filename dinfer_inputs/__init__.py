"""Seeded synthetic inputs for the block-denoising step: weights, token ids, masks, page tables.

This package holds no arithmetic of the decoding method.  It produces the
bit-reproducible random tensors that both the CPU oracle and the HIP path are
fed with, and the shape presets of the benchmark configurations.
"""
from .generator import (  # noqa: F401
    mix64,
    stream_key,
    normal,
    uniform_ids,
    bernoulli_bits,
)
from .configs import (  # noqa: F401
    ModelConfig,
    Workload,
    BASE_SEED,
    TENSOR_NAMES,
    LAYER_TENSOR_NAMES,
    model_preset,
    workload_preset,
    tensor_shape,
    make_weights,
    make_workload_inputs,
    synthetic_prefix_kv,
    peaked_positions,
    bf16_to_f32,
    f32_to_bf16,
)
