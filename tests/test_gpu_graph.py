"""The forward under HIP graph capture: captured once, replayed several times with eager work in between, every replay
compared with the eager result.  A forward enqueues kernels only (no allocation, no memset node, no host
synchronisation), which is what makes it capturable; the variant on the library's own workspace is the one meant
for callers that cannot hand a workspace over."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moe_oracle as orc

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("static_ws", [False, True], ids=["caller_workspace", "library_workspace"])
def test_forward_captured_in_a_graph_replays_like_eager(static_ws):
    import gpu_harness as H
    import paper_2502_19811_amd as moe
    cfg = wl.MoEConfig("graph", T=600, H=512, F=768, E=8, k=2, act=wl.ACT_SWIGLU, S=4, seed=500)
    inp = wl.make_inputs(cfg, threads=4)
    ids, w = orc.route_topk(inp.logits, cfg.k)
    layer = H.GpuLayer(cfg, inp, ids, w)
    layer.forward()
    base = layer.results()
    assert base.status == 0
    ref = orc.moe_layer(inp.x, inp.W1, inp.W2, ids, w, cfg.act)
    a, b = H.error_metrics(base.out, ref)
    assert a <= H.REL_TOL and b <= H.REL_TOL

    out_g = torch.zeros_like(layer.out)

    def enqueue():
        if static_ws:
            moe.moe_layer_forward_static(layer.plan, layer.x, layer.ids, layer.w, layer.W1, layer.W2, cfg.act, out_g)
        else:
            moe.moe_layer_forward(layer.plan, layer.x, layer.ids, layer.w, layer.W1, layer.W2, cfg.act, out_g, layer.ws)

    enqueue()                       # once eagerly: whatever is set up on first use happens outside the capture
    torch.cuda.synchronize()
    print(f"capturing ({'library' if static_ws else 'caller'} workspace)", flush=True)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue()
    for rep in range(4):
        out_g.fill_(3.0)
        graph.replay()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(H.bf16_to_np(out_g), base.out)
        # the program's own eager work between replays: another routing on the same plan, then the first one again
        if rep == 1:
            ids2 = np.ascontiguousarray(ids[::-1])
            layer.ids.copy_(torch.from_numpy(ids2).cuda())
            layer.forward()
            torch.cuda.synchronize()
            layer.ids.copy_(torch.from_numpy(ids).cuda())
        print(f"  replay {rep} ok", flush=True)
    layer.close()
