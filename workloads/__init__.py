"""Seeded synthetic inputs for tensor-network linear layers.

This module only draws random numbers, scales them, rounds them to the storage
type and describes shapes. It holds none of the method's arithmetic (no
contraction, no dense rebuild, no matrix product) so that both the CPU oracle's
tests and the GPU path's tests can take their inputs from it without sharing
any computation.
"""
from .configs import (  # noqa: F401
    FORMAT_DENSE,
    FORMAT_TT,
    FORMAT_TR,
    FORMAT_TUCKER,
    FORMAT_NAMES,
    TNSpec,
    baseline_spec,
    make_tensors,
    make_x,
    round_to_dtype,
    bf16_bits,
    qwen3_32b_stack,
    stack_spec,
    SEED_BASE,
)
