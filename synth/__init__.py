"""Seeded synthetic inputs: model shapes, random-init weights, token streams, tree shapes.

This package only *generates inputs*.  It holds none of the method's arithmetic
(no forward pass, no acceptance rule): the CPU oracle and the HIP library both
receive the arrays produced here and share nothing else.
"""
from .configs import ModelConfig, Workload, PRESETS, preset
from .weights import make_weights, weight_names, round_to_bf16
from .tokens import make_tokens, make_uniforms
from .trees import make_tree, chain_tree, full_tree, TreeSpec

__all__ = [
    "ModelConfig", "Workload", "PRESETS", "preset",
    "make_weights", "weight_names", "round_to_bf16",
    "make_tokens", "make_uniforms", "make_tree", "chain_tree", "full_tree", "TreeSpec",
]
