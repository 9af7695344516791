"""Seeded synthetic MoE-layer workloads shared by the tests, the bench and the oracle.

This package draws random inputs only.  It contains none of the MoE layer's
arithmetic (no gating, routing, FFN or combine code), so the HIP path and the
CPU oracle can both consume it without sharing any part of the method.
"""
from .moe_inputs import (  # noqa: F401
    MoEWorkload,
    WORKLOADS,
    bf16_round,
    bf16_bits,
    make_layer,
    make_ring_stack,
    RingStackPool,
    zipf_masses,
)
