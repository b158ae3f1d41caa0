"""BrownoutMoE layer forward for MI355X (gfx950): thin Python face of libbrownout_moe.so."""
from .binding import (MoeError, RouteOut, alloc_route_out, alloc_workspace, config_of, init, latency_p90, lib,
                      make_config, moe_build_united, moe_config, moe_distill_united, moe_forward, moe_route,
                      moe_route_static, pack_gate, probe_hbm_read, probe_mfma, profile_collect, profile_disable,
                      profile_enable, salc_update, with_packed_gate, workspace_size)

__all__ = ["MoeError", "RouteOut", "alloc_route_out", "alloc_workspace", "config_of", "init", "latency_p90", "lib",
           "make_config", "moe_build_united", "moe_config", "moe_distill_united", "moe_forward", "moe_route",
           "moe_route_static", "pack_gate", "probe_hbm_read", "probe_mfma", "profile_collect", "profile_disable",
           "profile_enable", "salc_update", "with_packed_gate", "workspace_size"]
