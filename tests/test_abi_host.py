"""Host-side behaviour of the C ABI (no GPU needed): the library loads, exports what the header declares, validates
arguments and sizes workspaces."""
import ctypes as C
import os
import re

import pytest

import paper_2502_19811_amd as moe
from paper_2502_19811_amd import binding
from conftest import ROOT, read_golden

SEG8 = [0, 16, 32, 48, 64, 80, 96, 112, 128]


def test_library_exports_every_declared_symbol():
    lib = moe.load_library()
    header = open(os.path.join(ROOT, "include", "moe_gfx950.h")).read()
    declared = set(re.findall(r"^(?:int|size_t|int32_t|int64_t|const char \*)\s*(moe_[a-z0-9_]+)\(", header, flags=re.M))
    assert declared, "no declarations found"
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in the header but not exported"
    assert declared == set(binding.EXPORTS)


def test_status_strings():
    assert moe.moe_status_string(0) == "ok"
    for code in range(-6, 0):
        assert moe.moe_status_string(code) not in ("ok", "unknown status")
    assert moe.moe_status_string(-99) == "unknown status"


def _create(**kw):
    a = dict(T=128, H=256, F=512, E=4, k=2, S=8, act=moe.MOE_ACT_GELU, seg_offsets=SEG8)
    a.update(kw)
    return moe.moe_plan_create(**a)


def test_plan_create_and_options():
    plan = _create()
    assert moe.moe_plan_workspace_bytes(plan) > 256 * (512 + 256) * 2           # holds h [R,F] and Y [R,H], R = 256
    assert moe.moe_plan_get_option(plan, "tile_m") in (64, 128, 256)
    # defaults that come from measurements: no prefetching workgroups, deep operand rings for the short tiles
    assert moe.moe_plan_get_option(plan, "n_prefetch") == 0 and moe.moe_plan_get_option(plan, "deep_short_tiles") == 1
    assert moe.moe_plan_get_option(plan, "n_dm") == 0 and moe.moe_plan_get_option(plan, "layer1_order") == 0
    for key, val in [("tile_m", 128), ("n_dm", 7), ("layer0_order", 1), ("layer1_order", 2), ("layer1_order", 0), ("spin_limit", 1000),
                     ("phases", 3), ("n_cu", 64), ("large_schedule", 1), ("block_m", 8),
                     ("layer0_order", 2), ("layer0_waves", 4), ("expected_ingest_gbps", 50), ("weights_packed", 1), ("alias_experts", 1), ("handoff_fences", 1), ("fuse_layers", 1), ("publish_every", 4),
                     ("n_prefetch", 16), ("prefetch_ahead", 32), ("prefetch_behind", 0), ("deep_short_tiles", 0)]:
        moe.moe_plan_set_option(plan, key, val)
        assert moe.moe_plan_get_option(plan, key) == val
    for key, val in [("tile_m", 100), ("n_dm", -2), ("layer0_order", 3), ("layer0_order", -2), ("layer0_waves", 9), ("phases", 16), ("large_schedule", 2),
                     ("block_m", 0), ("block_m", 9), ("n_prefetch", 12), ("n_prefetch", 72), ("prefetch_ahead", -1), ("deep_short_tiles", 2), ("no_such_key", 1)]:
        with pytest.raises(moe.MoEError) as e:
            moe.moe_plan_set_option(plan, key, val)
        assert e.value.status == -1
    assert moe.moe_plan_max_tiles(plan) >= 256 // 128 + 4
    moe.moe_plan_destroy(plan)


@pytest.mark.parametrize("kw,status", [
    (dict(H=0), -1), (dict(k=5), -1), (dict(act=7), -1), (dict(seg_offsets=[0, 16, 32, 48, 64, 80, 96, 112, 127]), -1),
    (dict(seg_offsets=[0, 32, 16, 48, 64, 80, 96, 112, 128]), -1),
    (dict(H=200), -4), (dict(F=300), -4), (dict(E=300, k=2), -4), (dict(S=65, seg_offsets=[0] * 65 + [128]), -4),
    (dict(act=moe.MOE_ACT_SWIGLU, F=192), -4),
])
def test_plan_create_rejects(kw, status):
    with pytest.raises(moe.MoEError) as e:
        _create(**kw)
    assert e.value.status == status


def test_forward_argument_checks_happen_before_any_gpu_work():
    lib = moe.load_library()
    plan = _create()
    need = moe.moe_plan_workspace_bytes(plan)
    buf = C.create_string_buffer(4096)
    addr = (C.addressof(buf) + 255) & ~255           # a 256-byte aligned non-NULL pointer; never dereferenced
    args = [plan, addr, addr, addr, addr, addr, moe.MOE_ACT_GELU, addr, addr, need, None, 0, None]
    bad = list(args); bad[1] = None
    assert lib.moe_layer_forward(*bad) == -1          # NULL x
    bad = list(args); bad[6] = moe.MOE_ACT_SWIGLU
    assert lib.moe_layer_forward(*bad) == -2          # act differs from the plan
    bad = list(args); bad[9] = need - 1
    assert lib.moe_layer_forward(*bad) == -3          # workspace too small
    bad = list(args); bad[1] = addr + 2
    assert lib.moe_layer_forward(*bad) == -1          # misaligned x
    bad = list(args); bad[8] = addr + 16
    assert lib.moe_layer_forward(*bad) == -1          # workspace not 256-byte aligned
    moe.moe_plan_destroy(plan)


def test_timing_calls_without_recorded_forwards():
    plan = _create()
    assert moe.moe_plan_forward_times(plan) == []
    ms, n = moe.moe_plan_phase_times(plan)
    assert n == 0 and ms == [0.0] * 4
    lib = moe.load_library()
    assert lib.moe_plan_forward_times(plan, None, 4, None) == -1
    moe.moe_plan_destroy(plan)


def test_workspace_grows_with_the_batch_and_holds_both_intermediates():
    sizes = []
    for T in (128, 256, 1024):
        plan = _create(T=T, seg_offsets=[T * i // 8 for i in range(9)])
        sizes.append(moe.moe_plan_workspace_bytes(plan))
        assert sizes[-1] >= 2 * T * (512 + 256) * 2      # h [R,F] and Y [R,H] in bf16, R = 2T
        moe.moe_plan_destroy(plan)
    assert sizes == sorted(sizes) and len(set(sizes)) == 3


def test_receive_buffer_bytes_table3():
    for M, N, mb in [[int(v) for v in r] for r in read_golden("table3_buffer_mb.txt")]:
        assert moe.moe_receive_buffer_bytes(M, N) == mb << 20


def test_empty_batch_plan():
    plan = _create(T=0, seg_offsets=[0] * 9)
    assert moe.moe_plan_workspace_bytes(plan) > 0
    moe.moe_plan_destroy(plan)


def test_static_forward_and_packing_argument_checks_happen_on_the_host():
    lib = moe.load_library()
    buf = C.create_string_buffer(4096)
    addr = (C.addressof(buf) + 255) & ~255           # aligned, non-NULL, never dereferenced
    # a plan whose workspace exceeds the library's fixed 32 MiB is refused before anything touches the GPU
    big = _create(T=8192, H=4096, F=14336, E=8, k=2, act=moe.MOE_ACT_SWIGLU, seg_offsets=[1024 * i for i in range(9)])
    assert moe.moe_plan_workspace_bytes(big) > 32 << 20
    assert lib.moe_layer_forward_static(big, addr, addr, addr, addr, addr, moe.MOE_ACT_SWIGLU, addr, None, 0, None) == -3
    assert lib.moe_layer_forward_static(None, addr, addr, addr, addr, addr, moe.MOE_ACT_SWIGLU, addr, None, 0, None) == -1
    # packing: both pointers of a pair or neither, aligned, not in place
    assert lib.moe_pack_weights(big, addr, None, None, None, None) == -1       # source without destination
    assert lib.moe_pack_weights(big, addr, None, addr, None, None) == -1       # in place
    assert lib.moe_pack_weights(big, addr, None, addr + 2, None, None) == -1   # misaligned destination
    assert lib.moe_pack_weights(None, addr, None, addr + 256, None, None) == -1
    assert lib.moe_pack_weights(big, None, None, None, None, None) == 0        # nothing to do is not an error
    moe.moe_plan_destroy(big)


def test_schedule_getter_sizes_and_argument_checks():
    lib = moe.load_library()
    plan = _create()                                  # T=128, H=256, F=512, GELU: 2 layer0 and 1 layer1 column tiles
    mt = moe.moe_plan_max_tiles(plan)
    assert moe.moe_plan_schedule_capacity(plan, 0) == mt * 2
    assert moe.moe_plan_schedule_capacity(plan, 1) == (mt + 24) * 1
    assert moe.moe_plan_schedule_capacity(plan, 2) == 0
    q = (C.c_int32 * 24)()
    assert lib.moe_get_schedule(plan, None, 0, None, q, None) == -1           # no workspace
    assert lib.moe_get_schedule(plan, C.addressof(q), 3, None, q, None) == -1  # no such layer
    moe.moe_plan_destroy(plan)


def test_layer0_waves_come_from_the_table_unless_set():
    seg = lambda T: [T * i // 8 for i in range(9)]
    # the three profiled shapes at the profiled rates (see default_layer0_waves)
    mixtral = _create(T=8192, H=4096, F=14336, E=8, k=2, act=moe.MOE_ACT_SWIGLU, seg_offsets=seg(8192))
    phi35 = _create(T=16384, H=4096, F=6400, E=16, k=2, act=moe.MOE_ACT_SWIGLU, seg_offsets=seg(16384))
    qwen2 = _create(T=4096, H=3584, F=2560, E=64, k=8, act=moe.MOE_ACT_SWIGLU, seg_offsets=seg(4096))
    expect = {mixtral: {0: 4, 25: 4, 50: 4, 100: 4, 200: 4}, phi35: {0: 4, 25: 8, 50: 4, 100: 4, 200: 4},
              qwen2: {0: 8, 25: 8, 50: 8, 100: 1, 200: 1}}
    for plan, table in expect.items():
        assert moe.moe_plan_get_option(plan, "layer0_order") == -1            # chosen per forward
        for gbps, waves in table.items():
            moe.moe_plan_set_option(plan, "expected_ingest_gbps", gbps)
            assert moe.moe_plan_get_option(plan, "layer0_waves") == waves, (gbps, waves)
    moe.moe_plan_set_option(mixtral, "layer0_waves", 7)                       # an explicit setting wins
    assert moe.moe_plan_get_option(mixtral, "layer0_waves") == 7
    for plan in expect:
        moe.moe_plan_destroy(plan)
    few = _create(S=2, seg_offsets=[0, 64, 128])
    assert moe.moe_plan_get_option(few, "layer0_waves") == 2                  # never more waves than segments
    moe.moe_plan_destroy(few)
