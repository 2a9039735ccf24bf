"""MI355X-native forward pass of one MoE layer: FP8 block-scaled expert GEMMs and Router Replay.

The product is the C-ABI library libmoe355.so (hand-written HIP kernels for
gfx950); this package only builds it, loads it and marshals arguments.
"""
from .binding import (EXPORTS, LIB_PATH, MoEError, load_library, moe_balance_lengths, moe_check_ids, moe_combine, moe_create,  # noqa: F401
                      moe_debug_copy_hidden, moe_probe_copy, moe_probe_fp8_mfma, moe_destroy, moe_profile_enable, moe_profile_read, moe_expert_ffn_fp8, moe_expert_ffn_fp8_gather, moe_quantize_fp8, moe_route,
                      moe_route_replay, moe_route_replay_ids, moe_route_replay_noalloc, moe_quantize_weights_fp8, moe_linear_fp8, moe_version)
from .layer import MoELayer  # noqa: F401
