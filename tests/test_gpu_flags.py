"""Ready flags, schedule orders and failure handling of the HIP path (GPU)."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moe_oracle as orc

pytestmark = pytest.mark.gpu


def _cfg():
    return wl.MoEConfig("flags", T=1024, H=512, F=768, E=8, k=2, act=wl.ACT_SWIGLU, S=8, seed=300)


def _setup(options=None, cfg=None):
    import gpu_harness as H
    cfg = cfg or _cfg()
    inp = wl.make_inputs(cfg, threads=4)
    ids, w = orc.route_topk(inp.logits, cfg.k)
    return H, cfg, inp, ids, w, H.GpuLayer(cfg, inp, ids, w, options or {})


def test_output_is_deterministic_and_independent_of_the_schedule():
    H, cfg, inp, ids, w, layer = _setup()
    layer.forward(); base = layer.results(); layer.close()
    ref = orc.moe_layer(inp.x, inp.W1, inp.W2, ids, w, cfg.act)
    a, b = H.error_metrics(base.out, ref)
    assert a <= H.REL_TOL and b <= H.REL_TOL
    for opts in ({}, {"layer0_order": 1}, {"layer1_order": 1}, {"layer1_order": 1, "n_dm": 16}, {"tile_m": 128},
                 {"n_cu": 64}, {"layer0_order": 2, "layer0_waves": 4}, {"layer0_order": 2, "layer0_waves": 8, "layer1_order": 1}):
        print(f"options {opts}", flush=True)
        _, _, _, _, _, l2 = _setup(opts)
        l2.forward(); r2 = l2.results(); l2.close()
        assert r2.status == 0
        # every output element is the same sum in the same order whatever the tiling and schedule
        np.testing.assert_array_equal(r2.out, base.out)
        np.testing.assert_array_equal(r2.perm, base.perm)


@pytest.mark.parametrize("opts", [{}, {"layer0_order": 1}, {"layer1_order": 1}, {"large_schedule": 1},
                                  {"large_schedule": 1, "layer0_order": 1}, {"tile_m": 64, "block_m": 2},
                                  {"layer0_order": 2, "layer0_waves": 8}, {"layer0_order": 2, "layer0_waves": 3},
                                  {"layer0_order": 2, "layer0_waves": 2, "tile_m": 64, "block_m": 3},
                                  {"large_schedule": 1, "layer0_order": 2}],
                         ids=lambda o: "-".join(f"{k}{v}" for k, v in o.items()) or "default")
def test_schedules_list_every_tile_once_in_the_documented_order(opts):
    """The device-built schedules read back: once-only, records equal to the tile table, segment order for the
    source-ordered layer0 list (Fig. 5) and panel-group order for the column-wise layer1 list (Fig. 6)."""
    H, cfg, inp, ids, w, layer = _setup(dict(opts, phases=1))
    layer.forward()
    run = layer.results()
    assert run.status == 0
    n0 = cfg.F // (128 if cfg.act == wl.ACT_SWIGLU else 256)
    n1 = cfg.H // 256
    items0, q0 = layer.schedule(0)
    items1, q1 = layer.schedule(1)
    layer.close()
    large = opts.get("large_schedule") == 1
    order0 = opts.get("layer0_order", 0)
    H.check_schedule(items0, q0, run.tiles, n0, seg_major=order0 == 1 or (order0 == 2 and large),
                     waves=(opts["layer0_waves"], cfg.S) if order0 == 2 and not large else None)
    H.check_schedule(items1, q1, run.tiles, n1, panel_major=opts.get("layer1_order") == 1)


def test_wave_order_with_many_segments_and_uneven_experts():
    """64 source segments of unequal size grouped into 8 and 5 waves, experts of very different load: the queues keep
    their invariants and the output its bits."""
    import gpu_harness as H
    cfg = wl.MoEConfig("waves64", T=3000, H=256, F=256, E=16, k=4, act=wl.ACT_SWIGLU, S=64, seed=302, skew_zipf=1.2,
                       dirichlet_segments=True)
    inp = wl.make_inputs(cfg, threads=4)
    ids, w = orc.route_topk(inp.logits, cfg.k)
    base_layer = H.GpuLayer(cfg, inp, ids, w, {"tile_m": 128})
    base_layer.forward(); base = base_layer.results(); base_layer.close()
    a, b = H.error_metrics(base.out, orc.moe_layer(inp.x, inp.W1, inp.W2, ids, w, cfg.act))
    assert a <= H.REL_TOL and b <= H.REL_TOL
    for n_waves in (8, 5):
        layer = H.GpuLayer(cfg, inp, ids, w, {"tile_m": 128, "layer0_order": 2, "layer0_waves": n_waves})
        layer.forward(); run = layer.results()
        assert run.status == 0
        items0, q0 = layer.schedule(0)
        items1, q1 = layer.schedule(1)
        layer.close()
        H.check_schedule(items0, q0, run.tiles, cfg.F // 128, waves=(n_waves, cfg.S))
        H.check_schedule(items1, q1, run.tiles, cfg.H // 256)
        np.testing.assert_array_equal(run.out, base.out)


def test_segment_boundaries_do_not_change_the_result():
    H, cfg, inp, ids, w, layer = _setup()
    layer.forward(); base = layer.results(); layer.close()
    other = wl.scaled(cfg, S=3)
    inp2 = wl.MoEInputs(other, inp.x, inp.W1, inp.W2, inp.logits, np.array([0, 100, 100, 1024], np.int32))
    l2 = H.GpuLayer(other, inp2, ids, w)
    l2.forward(); r2 = l2.results(); l2.close()
    np.testing.assert_array_equal(r2.out, base.out)
    np.testing.assert_array_equal(r2.perm, base.perm)
    assert set(r2.tiles["ready_seg"].tolist()) <= {0, 2}      # the empty segment 1 owns no row


def test_flags_arriving_late_and_out_of_order():
    # 64 of the compute units stay free for the flag writes of the side stream; the spin limit turns a lost flag into
    # an error instead of a hang
    H, cfg, inp, ids, w, layer = _setup({"n_cu": 128, "spin_limit": 1 << 24})
    layer.forward(); base = layer.results()
    flags = torch.zeros(cfg.S, dtype=torch.int32, device="cuda")
    host_vals = torch.full((cfg.S,), 7, dtype=torch.int32).pin_memory()
    torch.cuda.synchronize()
    layer.out.zero_()
    side = torch.cuda.Stream()
    main = torch.cuda.current_stream()
    print("forward waiting on flags", flush=True)
    layer.forward(seg_ready=flags, epoch=7, stream=main)
    with torch.cuda.stream(side):
        for s in [3, 0, 7, 1, 6, 2, 5, 4]:
            torch.cuda._sleep(2_000_000)                     # roughly a millisecond between arrivals
            flags[s:s + 1].copy_(host_vals[s:s + 1], non_blocking=True)
    side.synchronize()
    run = layer.results()
    layer.close()
    assert run.status == 0
    np.testing.assert_array_equal(run.out, base.out)


def test_missing_flag_times_out_instead_of_hanging():
    H, cfg, inp, ids, w, layer = _setup({"n_cu": 128, "spin_limit": 2000})
    flags = torch.full((cfg.S,), 5, dtype=torch.int32, device="cuda")
    flags[cfg.S - 1] = 4                                      # the last segment never reaches epoch 5
    print("forward with a flag that never arrives", flush=True)
    layer.forward(seg_ready=flags, epoch=5)
    run = layer.results()
    assert run.status == -6                                   # MOE_ERR_TIMEOUT, reported by the kernels
    # the same plan and workspace work again once the flag is there
    flags[cfg.S - 1] = 5
    layer.forward(seg_ready=flags, epoch=5)
    run2 = layer.results()
    layer.close()
    assert run2.status == 0
    ref = orc.moe_layer(inp.x, inp.W1, inp.W2, ids, w, cfg.act)
    a, b = H.error_metrics(run2.out, ref)
    assert a <= H.REL_TOL and b <= H.REL_TOL


def test_empty_batch_and_empty_experts():
    import gpu_harness as H
    import paper_2502_19811_amd as moe
    plan = moe.moe_plan_create(0, 256, 256, 4, 2, 2, moe.MOE_ACT_GELU, [0, 0, 0])
    z = torch.zeros(256, dtype=torch.uint8, device="cuda")
    ws = torch.zeros(max(256, moe.moe_plan_workspace_bytes(plan)), dtype=torch.uint8, device="cuda")
    moe.moe_layer_forward(plan, z, z, z, z, z, moe.MOE_ACT_GELU, z, ws)      # T = 0: nothing to do, no error
    moe.moe_plan_destroy(plan)
    # all tokens to experts 1 and 2 of 6: four experts receive no row at all
    cfg = wl.MoEConfig("hole", T=90, H=256, F=256, E=6, k=2, act=wl.ACT_GELU, S=2, seed=301)
    inp = wl.make_inputs(cfg, threads=2)
    ids = np.tile(np.array([[1, 2]], np.int32), (cfg.T, 1))
    w = np.tile(np.array([[0.75, 0.25]], np.float32), (cfg.T, 1))
    layer = H.GpuLayer(cfg, inp, ids, w)
    layer.forward(); run = layer.results(); layer.close()
    assert run.counts.tolist() == [0, 90, 90, 0, 0, 0]
    a, b = H.error_metrics(run.out, orc.moe_layer(inp.x, inp.W1, inp.W2, ids, w, cfg.act))
    assert a <= H.REL_TOL and b <= H.REL_TOL


def test_paced_arrival_by_a_producer_workgroup():
    """The peers' stand-in fills the receive buffer segment by segment while the layer runs; same bits as resident."""
    import paper_2502_19811_amd as moe
    H, cfg, inp, ids, w, layer = _setup({"n_cu": 128, "spin_limit": 1 << 26, "layer0_order": 1})
    layer.forward(); base = layer.results()
    staging = layer.x.clone()
    layer.x.zero_()
    layer.out.zero_()
    flags = torch.zeros(cfg.S, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    print("producer + forward", flush=True)
    counters = torch.zeros(cfg.S, dtype=torch.int32, device="cuda")
    moe.moe_play_arrival(layer.plan, staging, layer.x, flags, counters, 3, 2.0, 3, side)   # 1 MB at 2 GB/s: 0.5 ms
    layer.forward(seg_ready=flags, epoch=3)
    side.synchronize()
    run = layer.results()
    layer.close()
    assert run.status == 0
    assert flags.cpu().tolist() == [3] * cfg.S and counters.cpu().tolist() == [0] * cfg.S
    np.testing.assert_array_equal(run.out, base.out)


@pytest.mark.parametrize("order", [-1, 1, 0, 2])
def test_few_workgroups_walk_many_flagged_tiles(order):
    """8 workgroups take the 48 layer0 items of the source-ordered schedule one after the other while a paced producer
    raises the segment flags: a workgroup walks from a tile whose segment is there into successors whose segments
    are not (no early start, blocking wait) and into ones that are (early start under flags).  Same bits as resident."""
    import paper_2502_19811_amd as moe
    opts = {"n_cu": 8, "spin_limit": 1 << 26}
    if order >= 0:
        opts["layer0_order"] = order            # -1: no option set, the forward chooses (waves, because of the flags)
    H, cfg, inp, ids, w, layer = _setup(opts)
    layer.forward(); base = layer.results()
    staging = layer.x.clone()
    layer.x.zero_()
    layer.out.zero_()
    flags = torch.zeros(cfg.S, dtype=torch.int32, device="cuda")
    counters = torch.zeros(cfg.S, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    print(f"producer + 8-workgroup forward, layer0_order {order}", flush=True)
    # 1 MB at 1 GB/s: a millisecond of arrivals against about 0.3 ms of layer0 work per workgroup
    moe.moe_play_arrival(layer.plan, staging, layer.x, flags, counters, 9, 1.0, 2, side)
    layer.forward(seg_ready=flags, epoch=9)
    side.synchronize()
    run = layer.results()
    layer.close()
    assert run.status == 0
    assert flags.cpu().tolist() == [9] * cfg.S
    np.testing.assert_array_equal(run.out, base.out)


def test_measurement_options_do_what_they_say():
    """handoff_fences only adds memory fences (same bits); alias_experts makes every expert compute with expert 0's
    weights (checked against the oracle fed with those weights)."""
    H, cfg, inp, ids, w, layer = _setup()
    layer.forward(); base = layer.results(); layer.close()
    _, _, _, _, _, fenced = _setup({"handoff_fences": 1})
    fenced.forward(); r1 = fenced.results(); fenced.close()
    assert r1.status == 0
    np.testing.assert_array_equal(r1.out, base.out)
    _, _, _, _, _, aliased = _setup({"alias_experts": 1})
    aliased.forward(); r2 = aliased.results(); aliased.close()
    assert r2.status == 0
    W1a = np.ascontiguousarray(np.broadcast_to(inp.W1[:1], inp.W1.shape))
    W2a = np.ascontiguousarray(np.broadcast_to(inp.W2[:1], inp.W2.shape))
    a, b = H.error_metrics(r2.out, orc.moe_layer(inp.x, W1a, W2a, ids, w, cfg.act))
    assert a <= H.REL_TOL and b <= H.REL_TOL
    np.testing.assert_array_equal(r2.perm, base.perm)


def test_device_probes_report_plausible_ceilings():
    import torch
    import paper_2502_19811_amd as moe
    scratch = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    rnd = moe.moe_probe_mfma(True, 4000, scratch)
    zer = moe.moe_probe_mfma(False, 4000, scratch)
    print(f"mfma loop: random {rnd:.0f} TFLOP/s, zeros {zer:.0f} TFLOP/s", flush=True)
    assert 500.0 < rnd < 2600.0 and 500.0 < zer < 2600.0      # below the 2.5 PFLOP/s the data sheet states
    src = torch.arange(1 << 24, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    gbps = moe.moe_probe_copy(dst, src)
    print(f"copy: {gbps:.0f} GB/s", flush=True)
    assert torch.equal(dst, src) and 500.0 < gbps < 8000.0
    big = torch.zeros(8 << 20, dtype=torch.uint8, device="cuda")
    mix = moe.moe_probe_mix(7, 4000, big)                       # LDS reads, L2-resident loads, barrier
    print(f"mfma loop with a K step's data movement: {mix:.0f} TFLOP/s", flush=True)
    assert 300.0 < mix < 2600.0
    tf, ghz = moe.moe_probe_mix(7, 40000, big, with_clock=True)
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    busy = tf * 1e12 / (n_cu * 4 * ghz * 1e9 * 1024)           # a SIMD does 1024 flop per cycle with this instruction
    print(f"  core clock inside the loop {ghz:.2f} GHz, matrix cores busy {busy:.2f}", flush=True)
    assert 0.5 < ghz < 2.6 and 0.3 < busy < 1.05
    with pytest.raises(moe.MoEError):
        moe.moe_probe_mix(15, 4000, big)                        # streaming needs 4 MiB per compute unit
    with pytest.raises(moe.MoEError):
        moe.moe_probe_mfma(True, 0, scratch)
    with pytest.raises(moe.MoEError):
        moe.moe_probe_mfma(True, 100, torch.zeros(16, dtype=torch.uint8, device="cuda"))


def test_one_plan_and_workspace_serve_different_routings_in_a_row():
    """Nothing of a forward survives into the next one on the same plan and workspace: a second forward with another
    routing (other counts, other tile table, fewer tiles) and then the first routing again give what fresh runs give."""
    H, cfg, inp, ids, w, layer = _setup()
    layer.forward()
    first = layer.results()
    ref1 = orc.moe_layer(inp.x, inp.W1, inp.W2, ids, w, cfg.act)
    # second routing: everything to experts 0 and 5, uneven weights
    ids2 = np.tile(np.array([[5, 0]], np.int32), (cfg.T, 1))
    w2 = np.tile(np.array([[0.9, 0.1]], np.float32), (cfg.T, 1))
    layer.ids.copy_(torch.from_numpy(ids2).cuda())
    layer.w.copy_(torch.from_numpy(w2).cuda())
    layer.forward()
    second = layer.results()
    assert second.status == 0 and second.counts.tolist() == [cfg.T, 0, 0, 0, 0, cfg.T, 0, 0]
    a, b = H.error_metrics(second.out, orc.moe_layer(inp.x, inp.W1, inp.W2, ids2, w2, cfg.act))
    assert a <= H.REL_TOL and b <= H.REL_TOL
    layer.ids.copy_(torch.from_numpy(ids).cuda())
    layer.w.copy_(torch.from_numpy(w).cuda())
    layer.forward()
    third = layer.results()
    layer.close()
    np.testing.assert_array_equal(third.out, first.out)
    np.testing.assert_array_equal(third.perm, first.perm)
    a, b = H.error_metrics(third.out, ref1)
    assert a <= H.REL_TOL and b <= H.REL_TOL


def test_expert_ids_out_of_range_are_reported_and_harmless():
    """Ids outside [0, E) neither fault nor disturb other tokens: the forward reports them through the status word."""
    import paper_2502_19811_amd as moe
    H, cfg, inp, ids, w, layer = _setup()
    bad = ids.copy()
    bad_tokens = [3, 500, cfg.T - 1]
    bad[3, 0] = -1
    bad[500, 1] = cfg.E
    bad[cfg.T - 1, 0] = 1 << 20
    layer.ids.copy_(torch.from_numpy(bad).cuda())
    layer.forward()
    run = layer.results()
    assert run.status == -1 and moe.moe_status_string(run.status) == "invalid argument"
    assert int(run.counts.sum()) == cfg.R                       # every pair was routed somewhere
    good = np.setdiff1d(np.arange(cfg.T), bad_tokens)
    ref = orc.moe_layer_tokens(good, inp.x, inp.W1, inp.W2, ids, w, cfg.act)
    a, b = H.error_metrics(run.out[good], ref)
    assert a <= H.REL_TOL and b <= H.REL_TOL
    # the next forward with valid ids reports nothing
    layer.ids.copy_(torch.from_numpy(ids).cuda())
    layer.forward()
    assert layer.results().status == 0
    layer.close()
