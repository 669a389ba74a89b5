"""Seeded synthetic MoE-layer inputs.

This package only *draws numbers*: Gaussian tensors, bf16 bit patterns, planted routing
structure (biases, burst directions) and multinomial group sizes.  It contains none of the
layer's arithmetic (no logits, no top-k, no FFN) so that the CPU oracle and the HIP path can
both consume its buffers without sharing any code of the method itself.
"""
from .gen import (  # noqa: F401
    MoEShape,
    MoEInputs,
    bf16_bits_from_f32,
    gaussian_f32,
    gaussian_bf16_bits,
    expert_weights,
    tiny,
    mixtral,
    mixtral_skewed,
    fine_grained,
    ep_share_layer,
    ep_share_groups,
    custom,
    trace_steps,
    wide_few_experts,
    mid_grained,
    TRACE_CONSISTENT, TRACE_PAIR,
    MIXTRAL_D, MIXTRAL_F, MIXTRAL_E, MIXTRAL_K,
    EP_D, EP_F, EP_E, EP_K, EP_ELO, EP_ELOCAL,
)
