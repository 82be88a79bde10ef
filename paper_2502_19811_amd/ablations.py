"""Two timing ablations of the GroupGEMM kernels, through plan options that exist for measurement only.

1. Weight stream: the layer on plain weights, normally and with "alias_experts" (every expert reads expert 0's
   weights, so the weight stream stays in the caches while every other access is unchanged; results wrong on
   purpose).  The difference is what streaming the weights from HBM costs, i.e. the most any prefetching could gain.
2. Tile hand-off fences: the layer normally and with "handoff_fences" (an agent-scope release after every layer0
   tile, an agent-scope acquire before every layer1 tile; results unchanged).  The difference is what a tile-granular
   hand-off of h from layer0 tiles to layer1 tiles inside one launch would pay for memory ordering alone.

    python -m paper_2502_19811_amd.ablations --workload mixtral qwen2 qwen2_table2 mixtral_tp8
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", nargs="+", default=["mixtral", "qwen2", "qwen2_table2", "mixtral_tp8"])
    ap.add_argument("--steps", type=int, default=30)
    args = ap.parse_args()

    import numpy as np
    import torch

    import paper_2502_19811_amd as moe
    import workloads as wl

    for name in args.workload:
        cfg = wl.CONFIGS[name]
        inp = wl.make_inputs(cfg, threads=min(16, os.cpu_count() or 8))
        dev = lambda b: torch.from_numpy(b.view(np.int16)).cuda().view(torch.bfloat16)
        x, W1, W2 = dev(inp.x), dev(inp.W1), dev(inp.W2)
        ids = torch.zeros((cfg.T, cfg.k), dtype=torch.int32, device="cuda")
        w = torch.zeros((cfg.T, cfg.k), dtype=torch.float32, device="cuda")
        moe.moe_route_topk(torch.from_numpy(inp.logits).cuda(), cfg.k, ids, w)
        out = torch.zeros((cfg.T, cfg.H), dtype=torch.bfloat16, device="cuda")
        plan = moe.moe_plan_create(cfg.T, cfg.H, cfg.F, cfg.E, cfg.k, cfg.S, cfg.act, inp.seg_offsets.tolist())
        ws = torch.zeros(moe.moe_plan_workspace_bytes(plan), dtype=torch.uint8, device="cuda")

        def measure(option):
            """Mean layer0 / layer1 kernel time in us, two alternating rounds of normal and ablated runs."""
            acc = {0: [0.0, 0.0], 1: [0.0, 0.0]}
            for on in (0, 1, 0, 1):
                moe.moe_plan_set_option(plan, option, on)
                for _ in range(10):
                    moe.moe_layer_forward(plan, x, ids, w, W1, W2, cfg.act, out, ws)
                torch.cuda.synchronize()
                moe.moe_plan_set_option(plan, "profile", 1)
                for _ in range(args.steps):
                    moe.moe_layer_forward(plan, x, ids, w, W1, W2, cfg.act, out, ws)
                ms, _ = moe.moe_plan_phase_times(plan)
                moe.moe_plan_set_option(plan, "profile", 0)
                acc[on][0] += ms[1] * 500.0
                acc[on][1] += ms[2] * 500.0
            moe.moe_plan_set_option(plan, option, 0)
            return acc

        for option in ("alias_experts", "handoff_fences"):
            a = measure(option)
            print(json.dumps({"workload": name, "option": option,
                              "layer0_us": {"normal": round(a[0][0], 1), "with_option": round(a[1][0], 1),
                                            "change": round(a[1][0] / a[0][0] - 1, 3)},
                              "layer1_us": {"normal": round(a[0][1], 1), "with_option": round(a[1][1], 1),
                                            "change": round(a[1][1] / a[0][1] - 1, 3)}}), flush=True)
        moe.moe_plan_destroy(plan)
        del x, W1, W2, ws, out
        torch.cuda.empty_cache()
    return 0


if __name__ == "__main__":
    sys.exit(main())
