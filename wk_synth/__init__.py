"""Seeded synthetic inputs shaped like the paper's rollouts.

This module only *draws inputs*: random Q/K/V tensors with the intra-chunk
redundancy structure, looping camera trajectories and discrete action labels.
It holds none of the method's arithmetic (no similarity, no selection, no
retrieval distance, no attention) and is the only code that both the CPU
oracle's tests and the HIP path's tests/bench may share.

Shapes follow the paper: 880 tokens per latent frame for the Matrix-Game-2.0
shape and 1,560 for the LingBot-World-Fast shape (Sec. 1), chunks of F = 3
latent frames (Sec. 3), and trajectories that return to an earlier viewpoint
like the loop-closure benchmark of Sec. 5.1.
"""
from .configs import WkConfig, CONFIGS, get_config
from .generators import (
    normal,
    uniform,
    make_queries,
    make_native,
    make_chunk,
    make_revisit_keys,
    make_poses,
    make_action_labels,
    torch_dtype,
)

__all__ = [
    "WkConfig",
    "CONFIGS",
    "get_config",
    "normal",
    "uniform",
    "make_queries",
    "make_native",
    "make_chunk",
    "make_revisit_keys",
    "make_poses",
    "make_action_labels",
    "torch_dtype",
]
