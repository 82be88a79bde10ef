"""The forward that allocates nothing (moe_layer_forward_static, fixed workspace inside the library) against
moe_layer_forward on a caller-owned workspace: same bits, two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moe_oracle as orc

pytestmark = pytest.mark.gpu


def _run_both(cfg):
    import gpu_harness as H
    import paper_2502_19811_amd as moe
    inp = wl.make_inputs(cfg, threads=4)
    ids, w = orc.route_topk(inp.logits, cfg.k)
    layer = H.GpuLayer(cfg, inp, ids, w)
    layer.forward()
    expected = layer.results()
    assert expected.status == 0
    out_static = torch.zeros_like(layer.out)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    moe.moe_layer_forward_static(layer.plan, layer.x, layer.ids, layer.w, layer.W1, layer.W2, cfg.act, out_static)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before           # nothing went through torch's allocator either
    got = H.bf16_to_np(out_static)
    layer.close()
    ref = orc.moe_layer(inp.x, inp.W1, inp.W2, ids, w, cfg.act)
    a, b = H.error_metrics(got, ref)
    print(f"  {cfg.name}: static-workspace forward vs oracle {a:.3e} {b:.3e}", flush=True)
    assert a <= H.REL_TOL and b <= H.REL_TOL
    np.testing.assert_array_equal(got, expected.out)          # same kernels, same order of every sum


def test_static_workspace_forward_matches_the_workspace_forward_twice():
    big = wl.MoEConfig("static_a", T=1024, H=512, F=768, E=8, k=2, act=wl.ACT_SWIGLU, S=8, seed=400)
    small = wl.MoEConfig("static_b", T=301, H=256, F=512, E=4, k=2, act=wl.ACT_GELU, S=3, seed=401)
    print("static workspace, first call", flush=True)
    _run_both(big)
    print("static workspace, second call (smaller input, other activation)", flush=True)
    _run_both(small)


def test_static_workspace_refuses_plans_beyond_its_size():
    import paper_2502_19811_amd as moe
    cfg = wl.CONFIGS["mixtral"]
    plan = moe.moe_plan_create(cfg.T, cfg.H, cfg.F, cfg.E, cfg.k, cfg.S, cfg.act,
                               np.linspace(0, cfg.T, cfg.S + 1).astype(int).tolist())
    assert moe.moe_plan_workspace_bytes(plan) > 32 << 20
    z = torch.zeros(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(moe.MoEError) as e:
        moe.moe_layer_forward_static(plan, z, z, z, z, z, cfg.act, z)
    assert e.value.status == -3                               # MOE_ERR_WORKSPACE_TOO_SMALL, before anything is launched
    moe.moe_plan_destroy(plan)
