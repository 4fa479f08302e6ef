"""Seeded synthetic inputs for the unified-KV decode path.

This package only *draws inputs*: service shapes, context lengths, page
placement, and bf16 tensors.  It contains none of the attention or append
arithmetic, and it imports neither the oracle nor the HIP library, so both
sides of a parity test can be fed from it.
"""
from .workloads import (  # noqa: F401
    Service,
    Batch,
    PageStack,
    CONFIGS,
    SHAPES,
    make_config,
    make_batch,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    normal_bf16,
    lockstep_order,
    pages_for_tokens,
    to_split_layout,
    draw_prefill_inputs,
)
