"""BEAM binary-masked MoE layer forward for MI355X (gfx950).

`binding` exposes the C ABI of libbeam.so (include/beam.h) under the same
names; `synth` draws seeded synthetic layers; `build` compiles the library.
"""
from . import binding, synth  # noqa: F401
from .binding import (BEAM_BF16, BEAM_F32, BEAM_RULE_CUMPROB, BEAM_RULE_MASK, BEAM_WEIGHTS_PACKED, BEAM_WEIGHTS_PLAIN, BeamError, beam_abi_version, beam_block_workspace_bytes, beam_combine,  # noqa: F401
                      beam_expert_ffn, beam_fused_pair_row_bits, beam_mask_router_backward, beam_moe_block_forward, beam_moe_block_forward_timed, beam_moe_forward, beam_moe_forward_noalloc, beam_moe_forward_rule, beam_moe_forward_timed, beam_route_rule, beam_pack_weights, beam_permute, beam_probe_mfma, beam_probe_stream_read, beam_route_mask,
                      beam_status_string, beam_workspace_bytes, beam_workspace_logits_region, make_shape)
