"""Seeded synthetic workloads for the MoE-layer hot path.

This module only *draws inputs* (token embeddings, gate matrix, expert weights,
gate-bias tables) and rounds them to the storage dtype.  It contains none of the
method's arithmetic (no gating, planning, FFN or combine) and is the only code
shared by the CPU oracle's tests and the GPU path's tests / benchmark.
"""
from .generate import (CONFIGS, LayerInputs, bf16_bits, bf16_round,
                       from_bf16_bits, make_layer, make_stack, scaled)

__all__ = ["CONFIGS", "LayerInputs", "bf16_bits", "bf16_round",
           "from_bf16_bits", "make_layer", "make_stack", "scaled"]
