"""Seeded synthetic MoE-layer workloads.

This package holds shapes and random-number recipes only.  It contains none of
the MoE layer's arithmetic and is the one module that both the CPU oracle's
callers and the HIP path's callers may import.
"""
from .configs import MoEConfig, CONFIGS, get_config, capacity_from_factor
from .generate import BlockInputs, LayerInputs, make_block_inputs, make_inputs, make_logits

__all__ = [
    "MoEConfig", "CONFIGS", "get_config", "capacity_from_factor",
    "LayerInputs", "make_inputs", "make_logits", "BlockInputs", "make_block_inputs",
]
