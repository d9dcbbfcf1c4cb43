"""MI355X-native MoE-layer forward for TEAM-style block-diffusion decoding (C-ABI library + thin binding)."""
from .binding import (Config, TeamMoeError, make_config, status_string, team_moe_build_dispatch, team_moe_classify_tokens,
                      team_moe_combine,  # noqa: F401
                      team_moe_expert_ffn, team_moe_layer_forward, team_moe_layer_forward_rows, team_moe_layer_forward_two_round,
                      team_moe_layer_forward_unique_rows, team_moe_expert_ffn_w8, team_moe_layer_forward_w8,
                      team_moe_dequantize_w8, team_moe_layer_forward_ex, LayerArgs, team_moe_layer_forward_static, team_moe_workspace_status, internal_set, internal_get, internal_stream_read,
                      team_moe_route,
                      team_moe_route_two_round, team_moe_workspace_size)
