"""Seeded synthetic inputs shared by the tests, the benchmark and the oracle checks.

This package only *draws inputs*.  It holds none of the contrastive-loss
arithmetic: no logits, no softmax, no gradients.
"""
from .features import (  # noqa: F401
    ADVERSARIAL_KINDS,
    CONFIGS,
    WorkloadConfig,
    adversarial_pairs,
    bf16_bits_to_f32,
    clip_pairs,
    f32_to_bf16_bits,
    make_config_inputs,
    two_views,
)
