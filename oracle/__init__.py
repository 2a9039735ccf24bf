"""CPU oracle of the MoE-layer forward pass.  TEST INFRASTRUCTURE ONLY.

Plain numpy in float64; imported by tests/, the smoke check and the
benchmark's cpu_baseline leg, never by the product path.
"""
from . import fp_formats, moe_layer  # noqa: F401
