"""Sweep of the division point n_dm (data-movement workgroups of the layer1 kernel, Section 3.2.2 / Fig. 8).

    python -m paper_2502_19811_amd.split_sweep --workload mixtral qwen2 --n-dm 0 2 4 8 16 32

Prints, per workload, the layer1 kernel time (GroupGEMM + in-kernel combine) for every n_dm, and the time of the
variant with a separate combine kernel for comparison.
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
    ap.add_argument("--workload", nargs="+", default=["mixtral"])
    ap.add_argument("--n-dm", type=int, nargs="+", default=[0, 2, 4, 8, 16, 32])
    ap.add_argument("--steps", type=int, default=10)
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

        def measure(options):
            plan = moe.moe_plan_create(cfg.T, cfg.H, cfg.F, cfg.E, cfg.k, cfg.S, cfg.act, inp.seg_offsets.tolist())
            for k_, v_ in options.items():
                moe.moe_plan_set_option(plan, k_, v_)
            ws = torch.zeros(moe.moe_plan_workspace_bytes(plan), dtype=torch.uint8, device="cuda")
            for _ in range(3):
                moe.moe_layer_forward(plan, x, ids, w, W1, W2, cfg.act, out, ws)
            torch.cuda.synchronize()
            moe.moe_plan_set_option(plan, "profile", 1)
            for _ in range(args.steps):
                moe.moe_layer_forward(plan, x, ids, w, W1, W2, cfg.act, out, ws)
            ms, _ = moe.moe_plan_phase_times(plan)
            moe.moe_plan_destroy(plan)
            return ms

        rows = []
        for n_dm in args.n_dm:
            ms = measure({"layer1_order": 1, "n_dm": n_dm})
            rows.append({"workload": name, "n_dm": n_dm, "layer1_us": round(ms[2] * 1e3, 1),
                         "layer_us": round(sum(ms) * 1e3, 1)})
            print(json.dumps(rows[-1]), flush=True)
        ms = measure({"layer1_order": 0})
        print(json.dumps({"workload": name, "separate_combine_kernel": True,
                          "layer1_plus_combine_us": round((ms[2] + ms[3]) * 1e3, 1),
                          "layer_us": round(sum(ms) * 1e3, 1)}), flush=True)
        best = min(rows, key=lambda r: r["layer1_us"])
        print(json.dumps({"workload": name, "best_n_dm": best["n_dm"], "best_layer1_us": best["layer1_us"]}), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
