"""Seeded synthetic workloads shared by the tests, the benchmark and the smoke run.

This package only draws random tensors and names shapes.  It contains none of
the method's arithmetic, so both the CPU oracle's tests and the HIP path's
tests may consume it without sharing any computation.
"""
from .configs import CONFIGS, DRAFT_LAYERS, DraftLayerConfig, RoundConfig, get_config  # noqa: F401
from .generate import (  # noqa: F401
    SeededStream,
    make_attention_inputs,
    make_fp8_prefix,
    make_draft_weights,
    make_hidden_states,
    make_lm_head,
    make_prefix_lengths,
    make_target_logits,
    make_uniforms,
)
