"""Seeded synthetic inputs for the Talon hot path.

This package only makes inputs (random logits rows, Q/K/V tensors) and names the
workload shapes.  It holds none of the method's arithmetic: no softmax, no
ranking, no gating, no attention.  Both the CPU oracle's tests and the GPU
path's tests draw their inputs from here so that the two sides see identical
bytes.
"""
from .configs import CONFIGS, WorkloadConfig, get_config  # noqa: F401
from .staging import bf16_to_device, build_pool, root_tokens, to_device_logits  # noqa: F401
from .generators import (  # noqa: F401
    attention_inputs,
    bf16_bits_to_f64,
    f32_to_bf16_bits,
    logits_pool,
    logits_row,
    storage_to_f64,
    target_logits_pool,
    target_logits_row,
    zipf_row,
)
