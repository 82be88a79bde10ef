"""Arrival experiment on one GPU (the analogue of the paper's "communication latency hidden", Section 5.3).

A producer workgroup plays the peers: it copies the source segments of the receive buffer one after another at a
paced rate and raises each segment's ready flag.  The layer runs concurrently on another stream and starts every
layer0 tile as soon as the segment of its last row is there.  Reported per ingest rate and layer0 schedule:
the layer time with everything resident, the arrival time alone, the time of both together, and
hidden = 1 - (together - resident) / arrival.

    python -m paper_2502_19811_amd.arrival_experiment --workload mixtral --gbps 25 50 100
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
    ap.add_argument("--workload", default="mixtral")
    ap.add_argument("--gbps", type=float, nargs="+", default=[25.0, 50.0, 100.0])
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--free-cus", type=int, default=8, help="compute units left to the producer")
    ap.add_argument("--schedules", nargs="+", default=["0", "1", "2:8", "2:4", "2:2"],
                    help="layer0 schedules to compare: order or order:waves")
    args = ap.parse_args()

    import numpy as np
    import torch

    import paper_2502_19811_amd as moe
    import workloads as wl

    cfg = wl.CONFIGS[args.workload]
    inp = wl.make_inputs(cfg, threads=min(16, os.cpu_count() or 8))
    dev = lambda b: torch.from_numpy(b.view(np.int16)).cuda().view(torch.bfloat16)
    staging, W1, W2 = dev(inp.x), dev(inp.W1), dev(inp.W2)
    x = torch.zeros_like(staging)
    ids = torch.zeros((cfg.T, cfg.k), dtype=torch.int32, device="cuda")
    w = torch.zeros((cfg.T, cfg.k), dtype=torch.float32, device="cuda")
    moe.moe_route_topk(torch.from_numpy(inp.logits).cuda(), cfg.k, ids, w)
    out = torch.zeros((cfg.T, cfg.H), dtype=torch.bfloat16, device="cuda")
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count - args.free_cus
    main_s, side_s = torch.cuda.Stream(), torch.cuda.Stream()
    flags = torch.zeros(cfg.S, dtype=torch.int32, device="cuda")
    counters = torch.zeros(cfg.S, dtype=torch.int32, device="cuda")
    epoch = 0

    results = []
    for sched in args.schedules:
        order, _, waves = sched.partition(":")
        order, waves = int(order), int(waves or 0)
        plan = moe.moe_plan_create(cfg.T, cfg.H, cfg.F, cfg.E, cfg.k, cfg.S, cfg.act, inp.seg_offsets.tolist())
        moe.moe_plan_set_option(plan, "n_cu", n_cu)
        moe.moe_plan_set_option(plan, "layer0_order", order)
        moe.moe_plan_set_option(plan, "layer0_waves", waves)
        moe.moe_plan_set_option(plan, "spin_limit", 1 << 28)
        ws = torch.zeros(moe.moe_plan_workspace_bytes(plan), dtype=torch.uint8, device="cuda")

        def run(mode, gbps):
            """mode: 'resident' (x in place, no flags), 'arrival' (producer alone), 'both'."""
            nonlocal epoch
            ts = []
            for _ in range(args.reps + 1):
                epoch += 1
                if mode == "resident":
                    x.copy_(staging)
                torch.cuda.synchronize()
                e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
                e0.record(main_s)
                side_s.wait_event(e0)
                if mode in ("arrival", "both"):
                    moe.moe_play_arrival(plan, staging, x, flags, counters, epoch, gbps, args.free_cus, side_s)
                    e2.record(side_s)
                if mode in ("resident", "both"):
                    moe.moe_layer_forward(plan, x, ids, w, W1, W2, cfg.act, out, ws,
                                          flags if mode == "both" else None, epoch, main_s)
                main_s.wait_stream(side_s)
                e1.record(main_s)
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1) * 1e3)
                assert moe.moe_last_device_status(plan, ws, main_s) == 0 or mode == "arrival"
            return float(np.median(ts[1:]))

        resident = run("resident", 0)
        ref = out.clone()
        for gbps in args.gbps:
            arrival = run("arrival", gbps)
            both = run("both", gbps)
            assert torch.equal(out, ref), "output changed with staggered arrival"
            hidden = 1.0 - (both - resident) / arrival
            results.append({"workload": cfg.name, "layer0_order": order, "layer0_waves": waves, "ingest_GBps": gbps,
                            "resident_us": round(resident, 1), "arrival_alone_us": round(arrival, 1),
                            "together_us": round(both, 1), "hidden": round(hidden, 3), "n_cu": n_cu})
            print(json.dumps(results[-1]), flush=True)
        moe.moe_plan_destroy(plan)
    return 0


if __name__ == "__main__":
    sys.exit(main())
