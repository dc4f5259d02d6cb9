"""MI355X-native hot path of one GPU's share of an MoE layer's training step.

Thin Python binding over the C-ABI library libmoe_hip.so (declared in include/moe_hip.h).
Every step of the path runs in hand-written HIP kernels; PyTorch only provides device
memory and streams.  There is no CPU or PyTorch fallback: a missing library is an error.
"""
from .binding import (MoEShape, MoEHotPath, lib_path, load_library, moe_abi_version, moe_combine, moe_combine_bwd,
                      moe_dispatch, moe_dispatch_static, moe_route_dispatch, moe_route_dispatch_workspace_bytes, moe_route_aux_bwd, moe_dispatch_workspace_bytes, moe_expert_bwd, moe_expert_bwd_workspace_bytes,
                      moe_expert_fwd, moe_expert_fwd_workspace_bytes, moe_expert_fwd_gather, moe_expert_bwd_gather, moe_last_error, moe_route, moe_route_bwd, MoEError, moe_router_fwd, moe_router_bwd,
                      moe_router_fwd_workspace_bytes, moe_router_bwd_workspace_bytes,
                      moe_profile_enable, moe_profile_report, moe_copy_probe, moe_mfma_probe,
                      moe_aux_loss, moe_aux_loss_bwd, moe_aux_loss_workspace_bytes,
                      moe_plan_overlap_degree, moe_plan_predict_load, moe_plan_materialize, moe_plan_dispatch)

__all__ = ["MoEShape", "MoEHotPath", "MoEError", "lib_path", "load_library", "moe_abi_version", "moe_last_error",
           "moe_route", "moe_route_bwd", "moe_router_fwd", "moe_router_bwd", "moe_router_fwd_workspace_bytes",
           "moe_router_bwd_workspace_bytes", "moe_dispatch", "moe_dispatch_static", "moe_route_dispatch", "moe_route_dispatch_workspace_bytes", "moe_route_aux_bwd", "moe_expert_fwd", "moe_expert_fwd_gather", "moe_expert_bwd_gather", "moe_expert_bwd", "moe_combine", "moe_combine_bwd",
           "moe_profile_enable", "moe_profile_report", "moe_copy_probe", "moe_mfma_probe", "moe_dispatch_workspace_bytes", "moe_expert_fwd_workspace_bytes", "moe_expert_bwd_workspace_bytes",
           "moe_aux_loss", "moe_aux_loss_bwd", "moe_aux_loss_workspace_bytes",
           "moe_plan_overlap_degree", "moe_plan_predict_load", "moe_plan_materialize", "moe_plan_dispatch"]
