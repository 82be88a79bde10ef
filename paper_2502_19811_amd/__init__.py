"""MI355X-native MoE layer hot path: thin ctypes binding over libmoe_gfx950.so.

Every step of the path runs in the HIP kernels of the library; this module only marshals
arguments (torch tensors are used for device memory and streams).  There is no CPU fallback:
if the library has not been built, loading it raises.
"""
from .binding import (  # noqa: F401
    MOE_ACT_GELU,
    MOE_ACT_SWIGLU,
    MoEError,
    MoEShape,
    lib_path,
    load_library,
    moe_get_index_outputs,
    moe_get_schedule,
    moe_get_tile_table,
    moe_plan_schedule_capacity,
    moe_last_device_status,
    moe_layer_forward,
    moe_layer_forward_static,
    moe_pack_weights,
    moe_plan_create,
    moe_plan_destroy,
    moe_plan_get_option,
    moe_plan_max_tiles,
    moe_plan_forward_times,
    moe_plan_phase_times,
    moe_plan_set_option,
    moe_plan_workspace_bytes,
    moe_play_arrival,
    moe_probe_copy,
    moe_probe_mfma,
    moe_probe_mix,
    moe_receive_buffer_bytes,
    moe_route_topk,
    moe_status_string,
)
