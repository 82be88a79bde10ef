"""Where a GroupGEMM workgroup's time goes, tile by tile.

Builds the library once more with -DMOE_TILE_TRACE (into a temporary directory; the in-tree library has none of this
code), runs forwards back to back and reads back, for the last of them,, for every workgroup and tile, when the workgroup started on the tile, when
the operands of the first K step were in LDS, when the main loop ended and when the epilogue ended (100 MHz device
clock), and how many core cycles of the main loop its first wavefront spent at the synchronisation point of the K steps.  Prints per layer and tile height: the mean length of these three phases and of the gap to the next tile,
how far apart the workgroups start and finish, and how much of the launch a workgroup spends in main loops.

    python -m paper_2502_19811_amd.tile_trace --workload mixtral qwen2_table2
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

N_WG, N_SLOTS, N_WORDS = 256, 128, 6


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", nargs="+", default=["mixtral", "qwen2_table2"])
    ap.add_argument("--opt", action="append", default=[], help="plan option key=value")
    ap.add_argument("--forwards", type=int, default=20, help="forwards issued back to back; the last one is reported")
    args = ap.parse_args()

    if not os.environ.get("MOE_GFX950_LIB"):      # (set: a library already built with -DMOE_TILE_TRACE)
        from paper_2502_19811_amd import build
        tmp = tempfile.mkdtemp(prefix="moe_trace_")
        os.environ["MOE_GFX950_LIB"] = build.build_library(extra_flags=["-DMOE_TILE_TRACE"],
                                                           out_path=os.path.join(tmp, "libmoe_gfx950_trace.so"))
    import numpy as np
    import torch

    import paper_2502_19811_amd as moe
    import workloads as wl

    lib = moe.load_library()
    lib.moe_debug_tile_trace.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.moe_debug_tile_trace.restype = C.c_int

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
        W1p, W2p = torch.empty_like(W1), torch.empty_like(W2)
        moe.moe_pack_weights(plan, W1, W2, W1p, W2p)
        moe.moe_plan_set_option(plan, "weights_packed", 1)
        for kv in args.opt:
            k, v = kv.split("=")
            moe.moe_plan_set_option(plan, k, int(v))
        ws = torch.zeros(moe.moe_plan_workspace_bytes(plan), dtype=torch.uint8, device="cuda")
        for _ in range(5):
            moe.moe_layer_forward(plan, x, ids, w, W1p, W2p, cfg.act, out, ws)
        torch.cuda.synchronize()
        assert lib.moe_debug_tile_trace(1, None, None, None) == 0
        # forwards back to back, as a serving loop issues them; every launch notes its tiles over the previous one's,
        # so what is read back is the last forward, in the steady state of the board's clock control
        for _ in range(args.forwards):
            moe.moe_layer_forward(plan, x, ids, w, W1p, W2p, cfg.act, out, ws)
        torch.cuda.synchronize()
        stamps = np.zeros((2, N_WG, N_SLOTS, N_WORDS), dtype=np.uint64)
        kinds = np.zeros((2, N_WG, N_SLOTS), dtype=np.int32)
        counts = np.zeros((2, N_WG), dtype=np.int32)
        assert lib.moe_debug_tile_trace(0, stamps.ctypes.data, kinds.ctypes.data, counts.ctypes.data) == 0
        assert moe.moe_last_device_status(plan, ws) == 0
        us = stamps.astype(np.float64) / 100.0           # 100 MHz -> microseconds
        for layer in (0, 1):
            n = counts[layer]
            wgs = np.nonzero(n)[0]
            if len(wgs) == 0:
                continue
            first = np.array([us[layer, g, 0, 0] for g in wgs])
            last = np.array([us[layer, g, n[g] - 1, 3] for g in wgs])
            t_begin, t_end = first.min(), last.max()
            main_total = np.array([(us[layer, g, :n[g], 2] - us[layer, g, :n[g], 1]).sum() for g in wgs])
            res = {"workload": name, "layer": layer, "workgroups": int(len(wgs)), "tiles": int(n.sum()),
                   "tiles_per_workgroup_min_max": [int(n[wgs].min()), int(n[wgs].max())],
                   "launch_us": round(t_end - t_begin, 1),
                   "start_spread_us": round(first.max() - t_begin, 1),
                   "idle_at_end_us_mean_max": [round(float((t_end - last).mean()), 1), round(float((t_end - last).max()), 1)],
                   "share_of_launch_in_main_loops": round(float(main_total.mean() / (t_end - t_begin)), 3),
                   "truncated": bool((n >= N_SLOTS).any())}
            per_kind = {}
            for kind, label in ((2, "256"), (1, "128"), (0, "64")):
                for pre in (0, 1):
                    pro, mainl, epi, gap, sync, ghz = [], [], [], [], [], []
                    for g in wgs:
                        for i in range(n[g]):
                            if kinds[layer, g, i] != kind + 4 * pre:
                                continue
                            t = us[layer, g, i]
                            pro.append(t[1] - t[0]); mainl.append(t[2] - t[1]); epi.append(t[3] - t[2])
                            cyc = stamps[layer, g, i]
                            sync.append(float(cyc[5]) / max(float(cyc[4]), 1.0))
                            ghz.append(float(cyc[4]) / max(t[2] - t[1], 1e-3) / 1e3)
                            if i + 1 < n[g]:
                                gap.append(us[layer, g, i + 1, 0] - t[3])
                    if pro:
                        per_kind[f"{label} rows, {'early-started' if pre else 'cold start'}"] = {
                            "tiles": len(pro), "first_operands_us": round(float(np.mean(pro)), 2),
                            "main_loop_us": round(float(np.mean(mainl)), 2), "main_loop_p10_p90": [round(float(np.percentile(mainl, 10)), 2), round(float(np.percentile(mainl, 90)), 2)],
                            "main_loop_share_at_k_step_sync": round(float(np.mean(sync)), 3),
                            "main_loop_clock_ghz": round(float(np.mean(ghz)), 2),
                            "epilogue_us": round(float(np.mean(epi)), 2),
                            "gap_to_next_us": round(float(np.mean(gap)), 2) if gap else None}
            # core clock during the main loops of the 256-row tiles, by the tile's position in its workgroup's sequence
            by_index = []
            for i in range(int(n[wgs].max())):
                v = [float(stamps[layer, g, i, 4]) / max(us[layer, g, i, 2] - us[layer, g, i, 1], 1e-3) / 1e3
                     for g in wgs if i < n[g] and kinds[layer, g, i] % 4 == 2]
                if v:
                    by_index.append(round(float(np.mean(v)), 2))
            res["clock_ghz_by_tile_index"] = by_index
            res["per_tile"] = per_kind
            print(json.dumps(res), flush=True)
        moe.moe_plan_destroy(plan)
    return 0


if __name__ == "__main__":
    sys.exit(main())
