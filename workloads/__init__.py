"""Seeded synthetic workloads for the CTC-drafted speculative decoding step.

This package holds shapes and random input generation only.  It contains none of
the method's arithmetic: no projection, softmax, collapse, tree or attention code
lives here, so both the CPU oracle's tests and the HIP path's tests can draw the
same inputs from it without sharing any computation.
"""
from .configs import CONFIGS, StepConfig, get_config  # noqa: F401
from .generate import (  # noqa: F401
    AttentionCase,
    DraftLayerCase,
    StepInputs,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    make_attention_case,
    make_draft_layer_case,
    make_inputs,
    make_topk_case,
    round_to_storage,
)
