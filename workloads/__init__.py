"""Seeded synthetic MoE-layer workloads (inputs only).

This package draws the inputs of the MoE-layer forward pass: activations,
router weights, block-quantised expert weights and routing logs.  It is
used by the CPU oracle's tests and by the HIP path's tests and benchmark
alike, and it imports neither of them.
"""
from .configs import CONFIGS, MoEConfig, make_inputs, make_expert_weights, make_replay_log  # noqa: F401
