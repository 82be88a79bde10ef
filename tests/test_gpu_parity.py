"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moe_oracle as orc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import gpu_harness
    return gpu_harness


def _case(name, **kw):
    base = dict(T=128, H=256, F=512, E=4, k=2, act=wl.ACT_GELU, S=8, seed=100)
    base.update(kw)
    return wl.MoEConfig(name, **base)


SMALL_CASES = [
    wl.CONFIGS["tiny"],
    _case("ragged_swiglu", T=301, H=256, F=384, E=8, k=2, act=wl.ACT_SWIGLU, S=5, seed=101),
    _case("many_experts", T=200, H=512, F=256, E=64, k=8, act=wl.ACT_SWIGLU, S=8, seed=102),
    _case("one_expert", T=70, H=256, F=256, E=1, k=1, act=wl.ACT_GELU, S=1, seed=103),
    _case("single_token", T=1, H=256, F=256, E=4, k=2, act=wl.ACT_SWIGLU, S=2, seed=104),
    _case("wide_rows", T=700, H=768, F=640, E=3, k=3, act=wl.ACT_SWIGLU, S=8, seed=105),
    # the limits of the interface at once: 256 experts, 16 experts per token, 64 source segments
    _case("max_limits", T=96, H=256, F=128, E=256, k=16, act=wl.ACT_SWIGLU, S=64, seed=106),
    # GELU on full-height tiles (several per expert, ragged tail), and a second full-height SwiGLU case with k = 1
    _case("gelu_tall", T=1100, H=512, F=512, E=2, k=1, act=wl.ACT_GELU, S=4, seed=107),
    _case("swiglu_tall", T=900, H=256, F=256, E=2, k=1, act=wl.ACT_SWIGLU, S=3, seed=108),
    # more than 2048 M-tiles at tile_m = 64: the one-workgroup schedule builder is chosen by size
    _case("many_tiles", T=70000, H=256, F=128, E=4, k=2, act=wl.ACT_SWIGLU, S=8, seed=109),
]


def _check_index(run, cfg, ids, seg_offsets, tile_m):
    counts, offsets, perm, inv = orc.build_permutation(ids, cfg.E)
    np.testing.assert_array_equal(run.counts, counts)
    np.testing.assert_array_equal(run.offsets, offsets)
    np.testing.assert_array_equal(run.perm, perm)
    np.testing.assert_array_equal(run.inv_perm, inv)
    import gpu_harness
    gpu_harness.check_tile_table(run.tiles, cfg, offsets, perm, seg_offsets, tile_m)


@pytest.mark.parametrize("cfg", SMALL_CASES, ids=lambda c: c.name)
@pytest.mark.parametrize("tile_m", [64, 128, 256])
def test_layer_matches_oracle_small(H, cfg, tile_m):
    print(f"case {cfg.name} tile_m {tile_m}", flush=True)
    inp = wl.make_inputs(cfg, threads=4)
    ids, w = orc.route_topk(inp.logits, cfg.k)
    ref = orc.moe_layer(inp.x, inp.W1, inp.W2, ids, w, cfg.act)
    for l1 in (1, 0):
        layer = H.GpuLayer(cfg, inp, ids, w, {"tile_m": tile_m, "layer1_order": l1})
        layer.forward()
        run = layer.results()
        layer.close()
        assert run.status == 0
        _check_index(run, cfg, ids, inp.seg_offsets, tile_m)
        a, b = H.error_metrics(run.out, ref)
        print(f"  layer1_order {l1}: err {a:.3e} {b:.3e}", flush=True)
        assert a <= H.REL_TOL and b <= H.REL_TOL


@pytest.mark.parametrize("cfg", SMALL_CASES, ids=lambda c: c.name)
def test_packed_weights_give_the_same_bits(H, cfg):
    """The plan-time weight re-layout changes where the operands come from, not what is summed in which order."""
    print(f"packed case {cfg.name}", flush=True)
    inp = wl.make_inputs(cfg, threads=4)
    ids, w = orc.route_topk(inp.logits, cfg.k)
    ref = orc.moe_layer(inp.x, inp.W1, inp.W2, ids, w, cfg.act)
    for tile_m in (64, 128, 256):
        plain = H.GpuLayer(cfg, inp, ids, w, {"tile_m": tile_m})
        plain.forward(); base = plain.results(); plain.close()
        packed = H.GpuLayer(cfg, inp, ids, w, {"tile_m": tile_m}, packed=True)
        packed.forward(); run = packed.results(); packed.close()
        assert run.status == 0
        a, b = H.error_metrics(run.out, ref)
        print(f"  tile_m {tile_m}: err {a:.3e} {b:.3e}", flush=True)
        assert a <= H.REL_TOL and b <= H.REL_TOL
        np.testing.assert_array_equal(run.out, base.out)
        np.testing.assert_array_equal(run.perm, base.perm)


@pytest.mark.parametrize("cfg", SMALL_CASES, ids=lambda c: c.name)
def test_one_launch_for_both_groupgemms_gives_the_same_bits(H, cfg):
    """Layer0 and layer1 in one persistent launch, layer1 tiles waiting on per-M-tile counters: same output bit for bit
    as the two launches, for every tile height, with many and with few workgroups and with publication after every
    tile.  The small spin limit turns a lost hand-over into an error within milliseconds instead of a long wait."""
    print(f"one-launch case {cfg.name}", flush=True)
    inp = wl.make_inputs(cfg, threads=4)
    ids, w = orc.route_topk(inp.logits, cfg.k)
    for tile_m in (64, 128, 256):
        two = H.GpuLayer(cfg, inp, ids, w, {"tile_m": tile_m})
        two.forward(); base = two.results(); two.close()
        for extra in ({}, {"n_cu": 8, "publish_every": 1}, {"n_cu": 16, "publish_every": 3}):
            opts = dict(extra, tile_m=tile_m, fuse_layers=1, spin_limit=1 << 16)
            print(f"  {opts}", flush=True)
            one = H.GpuLayer(cfg, inp, ids, w, opts, packed=(tile_m == 128))
            one.forward(); run = one.results()
            assert run.status == 0
            np.testing.assert_array_equal(run.out, base.out)
            one.forward(); again = one.results(); one.close()      # counters start over on the same workspace
            assert again.status == 0
            np.testing.assert_array_equal(again.out, base.out)


@pytest.mark.parametrize("cfg", SMALL_CASES, ids=lambda c: c.name)
def test_reduction_in_the_layer1_epilogue_gives_the_same_bits(H, cfg):
    """layer1_order 2: the row that arrives last of a token's k reduces the token inside the layer1 epilogue.  Same
    bits as the separate combine kernel for k = 1, 2, 3, 8 and 16, every tile height, few and many workgroups, and
    together with the one-launch variant of the two GroupGEMMs."""
    print(f"epilogue-combine case {cfg.name}", flush=True)
    inp = wl.make_inputs(cfg, threads=4)
    ids, w = orc.route_topk(inp.logits, cfg.k)
    for tile_m in (64, 128, 256):
        sep = H.GpuLayer(cfg, inp, ids, w, {"tile_m": tile_m})
        sep.forward(); base = sep.results(); sep.close()
        for extra in ({}, {"n_cu": 8}, {"fuse_layers": 1, "spin_limit": 1 << 16}):
            opts = dict(extra, tile_m=tile_m, layer1_order=2)
            print(f"  {opts}", flush=True)
            layer = H.GpuLayer(cfg, inp, ids, w, opts)
            layer.out.fill_(7.0)                                  # every output row must be written by somebody
            layer.forward(); run = layer.results()
            assert run.status == 0
            np.testing.assert_array_equal(run.out, base.out)
            layer.forward(); again = layer.results(); layer.close()   # the arrival counters start over
            np.testing.assert_array_equal(again.out, base.out)


def test_router_matches_oracle(H):
    import paper_2502_19811_amd as moe
    for (T, E, k, seed) in [(128, 4, 2, 1), (513, 64, 8, 2), (100, 8, 8, 3), (77, 16, 1, 4), (64, 200, 6, 5)]:
        print(f"router T {T} E {E} k {k}", flush=True)
        g = wl.normal_f32((T, E), seed, 50, 1.0, threads=1)
        g[0, :] = 0.25                      # a row of exact ties: lowest expert ids win
        ids_ref, w_ref = orc.route_topk(g, k)
        ids = torch.zeros((T, k), dtype=torch.int32, device="cuda")
        w = torch.zeros((T, k), dtype=torch.float32, device="cuda")
        moe.moe_route_topk(torch.from_numpy(g).cuda(), k, ids, w)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(ids.cpu().numpy(), ids_ref)
        np.testing.assert_allclose(w.cpu().numpy(), w_ref, atol=2e-6)


@pytest.mark.parametrize("name", ["mixtral", "qwen2", "phi35", "skewed"])
def test_index_outputs_full_size(H, name):
    cfg = wl.CONFIGS[name]
    print(f"index build {name}", flush=True)
    inp = wl.make_inputs(cfg, threads=8, weights=False)
    ids, w = orc.route_topk(inp.logits, cfg.k)
    layer = H.GpuLayer(cfg, inp, ids, w, {"phases": 1})
    layer.forward()
    run = layer.results()
    import paper_2502_19811_amd as moe
    tile_m = moe.moe_plan_get_option(layer.plan, "tile_m")
    layer.close()
    assert run.status == 0
    _check_index(run, cfg, ids, inp.seg_offsets, tile_m)
    if name == "mixtral":
        # near-uniform load: close to the M*topk/E = 2048 rows per expert of Section 5.4
        assert abs(run.counts.mean() - 2048) < 1e-9 and run.counts.min() > 1800
    if name == "skewed":
        assert run.counts[0] / cfg.R > 0.3   # the popular expert takes about 40 % of the rows


@pytest.mark.parametrize("name", ["gelu_tall", "swiglu_tall", "wide_rows", "ragged_swiglu"])
def test_few_workgroups_walk_many_tiles(H, name):
    """With 8 workgroups every workgroup processes many tiles in a row, so the hand-over between tiles (the early
    start of a full-height successor included) is exercised for every kernel variant."""
    cfg = next(c for c in SMALL_CASES if c.name == name)
    inp = wl.make_inputs(cfg, threads=4)
    ids, w = orc.route_topk(inp.logits, cfg.k)
    ref = orc.moe_layer(inp.x, inp.W1, inp.W2, ids, w, cfg.act)
    for opts in ({"n_cu": 8}, {"n_cu": 8, "layer1_order": 1}, {"n_cu": 9, "tile_m": 128}):
        layer = H.GpuLayer(cfg, inp, ids, w, opts)
        layer.forward()
        run = layer.results()
        layer.close()
        assert run.status == 0
        a, b = H.error_metrics(run.out, ref)
        print(f"  {name} {opts}: err {a:.3e} {b:.3e}", flush=True)
        assert a <= H.REL_TOL and b <= H.REL_TOL
