"""Seeded synthetic inputs for the MoE-layer hot path.

This package holds input generation only: shapes, seeds, value distributions
and the one-time rounding of generated values to the storage dtype.  It holds
none of the method's arithmetic (no router, gating, FFN or combine), so both
the CPU oracle's tests and the HIP path's tests can draw the same bits from it
without sharing any code of the method itself.
"""
from .configs import MoEConfig, CONFIGS, get_config
from .synth import (
    bf16_bits_from_f32,
    make_layer,
    make_hidden,
    make_router,
    make_expert,
    make_residency_mask,
    make_prefetch_noise,
    tensor_seed,
)

__all__ = [
    "MoEConfig", "CONFIGS", "get_config",
    "bf16_bits_from_f32", "make_layer", "make_hidden", "make_router",
    "make_expert", "make_residency_mask", "make_prefetch_noise", "tensor_seed",
]
