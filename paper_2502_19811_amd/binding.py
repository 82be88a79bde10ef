"""ctypes binding with the same names as the C entry points of include/moe_gfx950.h.

Tensor arguments are torch tensors on the GPU (or None where the C call accepts NULL); only their
data pointers are passed on.  `stream` is a torch.cuda.Stream or None for the current stream.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

MOE_ACT_GELU = 0
MOE_ACT_SWIGLU = 1

_LIB_NAME = "libmoe_gfx950.so"
_lib = None

EXPORTS = [
    "moe_plan_create", "moe_plan_destroy", "moe_plan_set_option", "moe_plan_get_option",
    "moe_plan_workspace_bytes", "moe_plan_max_tiles", "moe_receive_buffer_bytes", "moe_route_topk",
    "moe_layer_forward", "moe_get_index_outputs", "moe_get_tile_table", "moe_last_device_status",
    "moe_status_string", "moe_plan_phase_times", "moe_plan_forward_times", "moe_play_arrival",
    "moe_probe_mfma", "moe_probe_copy", "moe_pack_weights", "moe_layer_forward_static", "moe_get_schedule",
    "moe_plan_schedule_capacity", "moe_probe_mix",
]


class MoEError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {moe_status_string(status)} ({status})")


class MoEShape(C.Structure):
    _fields_ = [("T", C.c_int32), ("H", C.c_int32), ("F", C.c_int32), ("E", C.c_int32), ("k", C.c_int32),
                ("S", C.c_int32), ("act", C.c_int32)]


def lib_path() -> str:
    """The in-tree library; MOE_GFX950_LIB names another build of the same sources (the measurement tools use it for
    builds with extra instrumentation)."""
    return os.environ.get("MOE_GFX950_LIB") or os.path.join(os.path.dirname(os.path.abspath(__file__)), _LIB_NAME)


def load_library():
    """Loads the built library.  Raises if it is missing: there is no other implementation to fall back to."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is not built; run `python -m paper_2502_19811_amd.build` "
                                f"(or __graft_entry__.build()) first")
    lib = C.CDLL(path)
    vp, i32p, f32p, u32p = C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p
    lib.moe_plan_create.argtypes = [C.POINTER(C.c_void_p), C.POINTER(MoEShape), C.POINTER(C.c_int32)]
    lib.moe_plan_create.restype = C.c_int
    lib.moe_plan_destroy.argtypes = [C.c_void_p]
    lib.moe_plan_destroy.restype = C.c_int
    lib.moe_plan_set_option.argtypes = [C.c_void_p, C.c_char_p, C.c_int64]
    lib.moe_plan_set_option.restype = C.c_int
    lib.moe_plan_get_option.argtypes = [C.c_void_p, C.c_char_p, C.POINTER(C.c_int64)]
    lib.moe_plan_get_option.restype = C.c_int
    lib.moe_plan_workspace_bytes.argtypes = [C.c_void_p]
    lib.moe_plan_workspace_bytes.restype = C.c_size_t
    lib.moe_plan_max_tiles.argtypes = [C.c_void_p]
    lib.moe_plan_max_tiles.restype = C.c_int32
    lib.moe_receive_buffer_bytes.argtypes = [C.c_int64, C.c_int64]
    lib.moe_receive_buffer_bytes.restype = C.c_size_t
    lib.moe_route_topk.argtypes = [f32p, C.c_int32, C.c_int32, C.c_int32, i32p, f32p, vp]
    lib.moe_route_topk.restype = C.c_int
    lib.moe_layer_forward.argtypes = [C.c_void_p, vp, i32p, f32p, vp, vp, C.c_int32, vp, vp, C.c_size_t, u32p,
                                      C.c_uint32, vp]
    lib.moe_layer_forward.restype = C.c_int
    lib.moe_layer_forward_static.argtypes = [C.c_void_p, vp, i32p, f32p, vp, vp, C.c_int32, vp, u32p, C.c_uint32, vp]
    lib.moe_layer_forward_static.restype = C.c_int
    lib.moe_get_index_outputs.argtypes = [C.c_void_p, vp, i32p, i32p, i32p, i32p, vp]
    lib.moe_get_index_outputs.restype = C.c_int
    lib.moe_get_schedule.argtypes = [C.c_void_p, vp, C.c_int32, i32p, C.POINTER(C.c_int32), vp]
    lib.moe_get_schedule.restype = C.c_int
    lib.moe_plan_schedule_capacity.argtypes = [C.c_void_p, C.c_int32]
    lib.moe_plan_schedule_capacity.restype = C.c_int64
    lib.moe_get_tile_table.argtypes = [C.c_void_p, vp, i32p, i32p, i32p, i32p, i32p, i32p, vp]
    lib.moe_get_tile_table.restype = C.c_int
    lib.moe_last_device_status.argtypes = [C.c_void_p, vp, vp]
    lib.moe_last_device_status.restype = C.c_int
    lib.moe_plan_phase_times.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.POINTER(C.c_int32)]
    lib.moe_plan_phase_times.restype = C.c_int
    lib.moe_plan_forward_times.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.c_int32, C.POINTER(C.c_int32)]
    lib.moe_plan_forward_times.restype = C.c_int
    lib.moe_probe_mfma.argtypes = [C.c_int32, C.c_int32, vp, C.c_size_t, C.POINTER(C.c_float), vp]
    lib.moe_probe_mfma.restype = C.c_int
    lib.moe_probe_mix.argtypes = [C.c_int32, C.c_int32, vp, C.c_size_t, C.POINTER(C.c_float), C.POINTER(C.c_float), vp]
    lib.moe_probe_mix.restype = C.c_int
    lib.moe_probe_copy.argtypes = [vp, vp, C.c_size_t, C.POINTER(C.c_float), vp]
    lib.moe_probe_copy.restype = C.c_int
    lib.moe_play_arrival.argtypes = [C.c_void_p, vp, vp, u32p, u32p, C.c_uint32, C.c_double, C.c_int32, vp]
    lib.moe_play_arrival.restype = C.c_int
    lib.moe_pack_weights.argtypes = [C.c_void_p, vp, vp, vp, vp, vp]
    lib.moe_pack_weights.restype = C.c_int
    lib.moe_status_string.argtypes = [C.c_int]
    lib.moe_status_string.restype = C.c_char_p
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream


def _check(status: int, where: str) -> None:
    if status != 0:
        raise MoEError(status, where)


def moe_status_string(status: int) -> str:
    return load_library().moe_status_string(status).decode()


def moe_plan_create(T: int, H: int, F: int, E: int, k: int, S: int, act: int, seg_offsets: Sequence[int]) -> int:
    """Returns the plan handle.  seg_offsets: S+1 host integers."""
    lib = load_library()
    shape = MoEShape(T, H, F, E, k, S, act)
    seg = (C.c_int32 * (S + 1))(*[int(v) for v in seg_offsets])
    handle = C.c_void_p()
    _check(lib.moe_plan_create(C.byref(handle), C.byref(shape), seg), "moe_plan_create")
    return handle.value


def moe_plan_destroy(plan: int) -> None:
    _check(load_library().moe_plan_destroy(plan), "moe_plan_destroy")


def moe_plan_set_option(plan: int, key: str, value: int) -> None:
    _check(load_library().moe_plan_set_option(plan, key.encode(), int(value)), f"moe_plan_set_option({key})")


def moe_plan_get_option(plan: int, key: str) -> int:
    v = C.c_int64()
    _check(load_library().moe_plan_get_option(plan, key.encode(), C.byref(v)), f"moe_plan_get_option({key})")
    return v.value


def moe_plan_workspace_bytes(plan: int) -> int:
    return load_library().moe_plan_workspace_bytes(plan)


def moe_plan_max_tiles(plan: int) -> int:
    return load_library().moe_plan_max_tiles(plan)


def moe_receive_buffer_bytes(M: int, N: int) -> int:
    return load_library().moe_receive_buffer_bytes(M, N)


def moe_route_topk(logits, k: int, topk_ids, topk_weights, stream=None) -> None:
    T, E = logits.shape
    _check(load_library().moe_route_topk(_ptr(logits), T, E, k, _ptr(topk_ids), _ptr(topk_weights), _stream(stream)),
           "moe_route_topk")


def moe_layer_forward(plan: int, x, topk_ids, topk_weights, W1, W2, act: int, out, workspace, seg_ready=None,
                      ready_epoch: int = 0, stream=None) -> None:
    _check(load_library().moe_layer_forward(plan, _ptr(x), _ptr(topk_ids), _ptr(topk_weights), _ptr(W1), _ptr(W2), act,
                                            _ptr(out), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                            _ptr(seg_ready), ready_epoch, _stream(stream)), "moe_layer_forward")


def moe_layer_forward_static(plan: int, x, topk_ids, topk_weights, W1, W2, act: int, out, seg_ready=None,
                             ready_epoch: int = 0, stream=None) -> None:
    """moe_layer_forward on the library's own fixed workspace (no allocation; plans up to 32 MiB of workspace)."""
    _check(load_library().moe_layer_forward_static(plan, _ptr(x), _ptr(topk_ids), _ptr(topk_weights), _ptr(W1), _ptr(W2),
                                                   act, _ptr(out), _ptr(seg_ready), ready_epoch, _stream(stream)),
           "moe_layer_forward_static")


def moe_pack_weights(plan: int, W1, W2, W1_packed, W2_packed, stream=None) -> None:
    _check(load_library().moe_pack_weights(plan, _ptr(W1), _ptr(W2), _ptr(W1_packed), _ptr(W2_packed), _stream(stream)),
           "moe_pack_weights")


def moe_get_index_outputs(plan: int, workspace, expert_counts=None, expert_offsets=None, perm=None, inv_perm=None,
                          stream=None) -> None:
    _check(load_library().moe_get_index_outputs(plan, _ptr(workspace), _ptr(expert_counts), _ptr(expert_offsets),
                                                _ptr(perm), _ptr(inv_perm), _stream(stream)), "moe_get_index_outputs")


def moe_get_tile_table(plan: int, workspace, n_tiles, tile_expert, tile_row0, tile_rows, tile_ready_seg,
                       tile_height=None, stream=None) -> None:
    _check(load_library().moe_get_tile_table(plan, _ptr(workspace), _ptr(n_tiles), _ptr(tile_expert), _ptr(tile_row0),
                                             _ptr(tile_rows), _ptr(tile_ready_seg), _ptr(tile_height),
                                             _stream(stream)),
           "moe_get_tile_table")


def moe_plan_schedule_capacity(plan: int, layer: int) -> int:
    return load_library().moe_plan_schedule_capacity(plan, layer)


def moe_get_schedule(plan: int, workspace, layer: int, items=None, stream=None):
    """Queues of the last forward's tile schedule: (first position, items, stride) per XCD; items (a device int32
    tensor [capacity, 8]) receives the item records."""
    q = (C.c_int32 * 24)()
    _check(load_library().moe_get_schedule(plan, _ptr(workspace), layer, _ptr(items), q, _stream(stream)),
           "moe_get_schedule")
    return [(q[x], q[8 + x], q[16 + x]) for x in range(8)]


def moe_last_device_status(plan: int, workspace, stream=None) -> int:
    return load_library().moe_last_device_status(plan, _ptr(workspace), _stream(stream))


def moe_plan_phase_times(plan: int):
    """(ms per phase [index build, layer0, layer1 (+fused combine), stand-alone combine], forwards averaged)."""
    ms = (C.c_float * 4)()
    n = C.c_int32()
    _check(load_library().moe_plan_phase_times(plan, ms, C.byref(n)), "moe_plan_phase_times")
    return [float(v) for v in ms], n.value


def moe_play_arrival(plan: int, staging, x, seg_ready, seg_counters, ready_epoch: int, gbytes_per_s: float,
                     n_workgroups: int = 1, stream=None) -> None:
    _check(load_library().moe_play_arrival(plan, _ptr(staging), _ptr(x), _ptr(seg_ready), _ptr(seg_counters),
                                           ready_epoch, float(gbytes_per_s), n_workgroups, _stream(stream)),
           "moe_play_arrival")


def moe_plan_forward_times(plan: int, capacity: int = 256):
    """ms of each forward recorded since the last moe_plan_phase_times call (needs the "profile" option)."""
    ms = (C.c_float * capacity)()
    n = C.c_int32()
    _check(load_library().moe_plan_forward_times(plan, ms, capacity, C.byref(n)), "moe_plan_forward_times")
    return [float(ms[i]) for i in range(n.value)]


def moe_probe_mfma(random_data, iters: int, scratch, stream=None) -> float:
    """TFLOP/s of the library's register-only bf16 MFMA loop on this device (scratch: a device tensor of >= 1 MiB).
    random_data: False zeros, True random operands, 2 random operands with the 16x16x32 instruction."""
    out = C.c_float()
    _check(load_library().moe_probe_mfma(int(random_data), iters, _ptr(scratch), scratch.numel() * scratch.element_size(),
                                         C.byref(out), _stream(stream)), "moe_probe_mfma")
    return float(out.value)


def moe_probe_mix(mode: int, iters: int, scratch, stream=None, with_clock: bool = False):
    """TFLOP/s of the MFMA loop with GroupGEMM-like data movement around it (mode bits: 1 LDS reads, 2 global->LDS
    loads, 4 barrier, 8 a quarter of the loads from HBM, 16 the 16x16x32 instruction); iters K steps; scratch: a device tensor, see the header for its size.
    with_clock: returns (TFLOP/s, core clock in GHz inside the loop)."""
    out, ghz = C.c_float(), C.c_float()
    _check(load_library().moe_probe_mix(mode, iters, _ptr(scratch), scratch.numel() * scratch.element_size(),
                                        C.byref(out), C.byref(ghz) if with_clock else None, _stream(stream)),
           "moe_probe_mix")
    return (float(out.value), float(ghz.value)) if with_clock else float(out.value)


def moe_probe_copy(dst, src, stream=None) -> float:
    """GB/s (read + written) of a plain device copy of src into dst."""
    out = C.c_float()
    nbytes = src.numel() * src.element_size()
    _check(load_library().moe_probe_copy(_ptr(dst), _ptr(src), nbytes, C.byref(out), _stream(stream)), "moe_probe_copy")
    return float(out.value)
