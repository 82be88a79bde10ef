#!/usr/bin/env python3
"""Benchmark of the fused MoE layer on one MI355X.

A step is one pass of the whole hot path (index build, layer0 GroupGEMM + activation, layer1 GroupGEMM with the
top-k combine) through moe_layer_forward on the Mixtral-8x7B-shaped synthetic workload, inputs resident in HBM.
Prints one JSON line: the layer's TFLOP/s (and µs, fraction of the bf16 MFMA peak), the roofline of the dominant
kernel (layer0 GroupGEMM) from HIP events recorded inside the timed steps, and the CPU oracle timed on a bounded
sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak (published)
METRIC = "fused MoE layer µs + TFLOP/s (fraction of bf16 MFMA peak) on 1 MI355X"


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="mixtral", help="tiny | mixtral | qwen2 | phi35 | skewed")
    ap.add_argument("--opt", action="append", default=[], help="plan option key=value (repeatable)")
    ap.add_argument("--packed", type=int, default=1, choices=[0, 1],
                    help="1 (default): the weights are re-laid out once, before the timed steps, with moe_pack_weights; "
                         "the layer is then also timed on the plain weights (10 steps, reported as plain_weights)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one forward in a HIP graph and time its replays (for launch-bound sizes such as the "
                         "tiny workload); the per-phase events are then not recorded")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=8192,
                    help="tokens the CPU oracle is timed (and the GPU output checked) on; 8192 is the whole default workload")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (reference point for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures the one-GPU share of the layer; --gpus above 1 is not part of this build "
              "(no collectives, no sharding)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2502_19811_amd as moe
    import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    moe.load_library()   # raises if the HIP library is not built: there is no fallback
    cfg = wl.CONFIGS[args.workload]
    threads = min(16, os.cpu_count() or 8)
    t0 = time.time()
    inp = wl.make_inputs(cfg, threads=threads)
    t_gen = time.time() - t0

    def dev_bf16(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)

    x, W1, W2 = dev_bf16(inp.x), dev_bf16(inp.W1), dev_bf16(inp.W2)
    logits = torch.from_numpy(inp.logits).cuda()
    ids = torch.zeros((cfg.T, cfg.k), dtype=torch.int32, device="cuda")
    w = torch.zeros((cfg.T, cfg.k), dtype=torch.float32, device="cuda")
    moe.moe_route_topk(logits, cfg.k, ids, w)          # the gate runs on the GPU too; it is outside the timed layer
    out = torch.zeros((cfg.T, cfg.H), dtype=torch.bfloat16, device="cuda")
    plan = moe.moe_plan_create(cfg.T, cfg.H, cfg.F, cfg.E, cfg.k, cfg.S, cfg.act, inp.seg_offsets.tolist())
    for kv in args.opt:
        key, val = kv.split("=")
        moe.moe_plan_set_option(plan, key, int(val))
    W1_plain, W2_plain = W1, W2
    if args.packed:
        W1p, W2p = torch.empty_like(W1), torch.empty_like(W2)
        moe.moe_pack_weights(plan, W1, W2, W1p, W2p)      # plan-time, outside the timed region
        torch.cuda.synchronize()
        W1, W2 = W1p, W2p
        del W1p, W2p
        moe.moe_plan_set_option(plan, "weights_packed", 1)
    ws = torch.zeros(moe.moe_plan_workspace_bytes(plan), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        moe.moe_layer_forward(plan, x, ids, w, W1, W2, cfg.act, out, ws, None, 0, stream)

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB read, 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            moe.moe_layer_forward(plan, x, ids, w, W1, W2, cfg.act, out, ws, None, 0, torch.cuda.current_stream())
        eager_step, step = step, graph.replay
        for _ in range(3):
            step()
        torch.cuda.synchronize()
    else:
        moe.moe_plan_set_option(plan, "profile", 1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    if args.graph:
        per_forward_us, n_dropped, phase_ms, n_prof = [], 0, [0.0] * 4, 0
        step = eager_step
    else:
        per_forward_us = sorted(v * 1e3 for v in moe.moe_plan_forward_times(plan, 256))
        n_dropped = moe.moe_plan_get_option(plan, "profile_dropped")
        phase_ms, n_prof = moe.moe_plan_phase_times(plan)
        moe.moe_plan_set_option(plan, "profile", 0)
    status = moe.moe_last_device_status(plan, ws)
    assert status == 0, f"device status {status}"

    ms_per_step = elapsed / args.steps * 1e3
    tflops = cfg.flops / (ms_per_step * 1e-3) / 1e12
    # dominant kernel: the layer0 GroupGEMM (2*R*H*F1 flop per launch, one launch per step)
    l0_flop = 2.0 * cfg.R * cfg.H * cfg.F1
    l1_flop = 2.0 * cfg.R * cfg.F * cfg.H
    l0_tflops = l0_flop / (phase_ms[1] * 1e-3) / 1e12 if phase_ms[1] > 0 else 0.0
    l1_tflops = l1_flop / (phase_ms[2] * 1e-3) / 1e12 if phase_ms[2] > 0 else 0.0
    # Bytes per launch of that kernel between the L2s and the memory side, from the committed rocprofv3 --pmc summary
    # (FETCH_SIZE + WRITE_SIZE, each scaled by what the counter reads for a plain 1 GiB copy); None if no summary
    # exists for this workload.  The counters sit at the L2s: reads served by the Infinity Cache are included, and
    # rocprofv3 offers no counter behind it on this device, so the HBM share cannot be separated.
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"group_gemm_{cfg.name}_pmc_traffic.md")
    if os.path.exists(tpath):
        for line in open(tpath):
            if line.startswith("l2_fabric_bytes_per_launch layer0:"):
                traffic = float(line.split(":")[1])

    # the same layer on the plain row-major weights, for comparison (not the headline: 10 steps)
    plain = None
    if args.packed:
        moe.moe_plan_set_option(plan, "weights_packed", 0)
        for _ in range(3):
            moe.moe_layer_forward(plan, x, ids, w, W1_plain, W2_plain, cfg.act, out, ws, None, 0, stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(10):
            moe.moe_layer_forward(plan, x, ids, w, W1_plain, W2_plain, cfg.act, out, ws, None, 0, stream)
        torch.cuda.synchronize()
        ms_plain = (time.perf_counter() - t1) / 10 * 1e3
        plain = {"us_per_layer": round(ms_plain * 1e3, 1), "tflops": round(cfg.flops / (ms_plain * 1e-3) / 1e12, 2),
                 "frac_of_bf16_peak": round(cfg.flops / (ms_plain * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4), "steps": 10}
        moe.moe_plan_set_option(plan, "weights_packed", 1)
        step()                              # the output checked below comes from the packed path
        torch.cuda.synchronize()

    result = {
        "metric": METRIC,
        "value": round(tflops, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "us_per_layer": round(ms_per_step * 1e3, 1),
        "frac_of_bf16_peak": round(tflops / PEAK_BF16_TFLOPS, 4),
        # per forward, from the events the library records on the stream (at most the last 64 forwards)
        "us_per_layer_min_median_p90": [round(per_forward_us[0], 1), round(per_forward_us[len(per_forward_us) // 2], 1),
                                        round(per_forward_us[min(len(per_forward_us) - 1, int(0.9 * len(per_forward_us)))], 1)]
        if per_forward_us else None,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={cfg.T} H={cfg.H} F={cfg.F} E={cfg.E} top{cfg.k} "
                               f"{'SwiGLU' if cfg.act == wl.ACT_SWIGLU else 'GELU'} S={cfg.S} seed={cfg.seed}",
                   "tile_m": moe.moe_plan_get_option(plan, "tile_m"), "n_dm": moe.moe_plan_get_option(plan, "n_dm"),
                   "layer1_order": moe.moe_plan_get_option(plan, "layer1_order"),
                   "weights_packed": moe.moe_plan_get_option(plan, "weights_packed"),
                   "hip_graph_replay": bool(args.graph),
                   "gather": "fused into layer0's operand loads (no separate phase, no materialised copy)",
                   "device": device_info(torch),
                   "flop_per_layer": cfg.flops, "input_generation_s": round(t_gen, 1)},
        "phases_us": {"index_build": round(phase_ms[0] * 1e3, 1), "layer0_gemm": round(phase_ms[1] * 1e3, 1),
                      "layer1_gemm": round(phase_ms[2] * 1e3, 1), "combine": round(phase_ms[3] * 1e3, 1),
                      "forwards_averaged": n_prof, "forwards_not_recorded": n_dropped, "layer1_tflops": round(l1_tflops, 1),
                      # the reduction reads k rows of Y per token (plus 8 index/weight bytes per row) and writes out
                      "combine_hbm_gbps": round((2.0 * cfg.R * cfg.H + 8.0 * cfg.R + 2.0 * cfg.T * cfg.H)
                                                / (phase_ms[3] * 1e-3) / 1e9, 1) if phase_ms[3] > 0 else None},
        "roofline": {"bound": "mfma", "kernel": "k_group_gemm layer0 (fc1 + activation)", "achieved": round(l0_tflops, 1),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(l0_tflops / PEAK_BF16_TFLOPS, 4),
                     "traffic": traffic,
                     "traffic_is": "bytes between the L2s and the memory side (FETCH_SIZE + WRITE_SIZE), Infinity Cache "
                                   "hits included; no HBM-level counter is available"},
        "plain_weights": plain,
    }

    # what this board sustains with the same MFMA instruction from registers, and its copy rate: context for the
    # fractions above (the published peak assumes a clock the board does not hold under this load)
    probe_scratch = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    copy_src = torch.ones(1 << 28, dtype=torch.uint8, device="cuda")
    copy_dst = torch.empty_like(copy_src)
    mfma_random = moe.moe_probe_mfma(True, 100000, probe_scratch)      # about 0.1 s of load: the clock settles
    result["device_ceilings"] = {
        "mfma_loop_random_bf16_tflops": round(mfma_random, 1),
        "mfma_loop_zeros_tflops": round(moe.moe_probe_mfma(False, 100000, probe_scratch), 1),
        "copy_gbps_read_plus_write": round(moe.moe_probe_copy(copy_dst, copy_src), 1),
        "layer_frac_of_mfma_loop_random": round(tflops / mfma_random, 4),
    }
    del copy_src, copy_dst

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, inp, ids.cpu().numpy(), w.cpu().numpy(), out, args.cpu_sample_tokens)
    print(json.dumps(result, ensure_ascii=False))
    moe.moe_plan_destroy(plan)
    return 0


def device_info(torch):
    """Name, compute units and maximum clock of the GPU, as the runtime reports them."""
    pr = torch.cuda.get_device_properties(0)
    info = {"name": pr.name, "compute_units": pr.multi_processor_count}
    clock_khz = getattr(pr, "clock_rate", None)
    if clock_khz:
        info["max_clock_mhz"] = round(clock_khz / 1e3)
    return info


def cpu_baseline(cfg, inp, ids, w, out_gpu, n_tokens):
    """The CPU oracle, as it stands, on an evenly spaced sample of tokens of the same workload."""
    import numpy as np
    from threadpoolctl import threadpool_info

    from oracle import moe_oracle as orc

    n = min(n_tokens, cfg.T)
    tokens = np.unique(np.linspace(0, cfg.T - 1, n).astype(np.int64))
    t0 = time.perf_counter()
    ref = orc.moe_layer_tokens(tokens, inp.x, inp.W1, inp.W2, ids, w, cfg.act)
    dt = time.perf_counter() - t0
    flop = cfg.flops * len(tokens) / cfg.T
    got = out_gpu[tokens].float().cpu().numpy().astype(np.float64)
    diff = np.abs(got - ref)
    rms = float(np.sqrt(np.mean(ref * ref)))
    cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return {"value": round(flop / dt / 1e12, 4), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": (f"all {cfg.T} tokens" if len(tokens) == cfg.T else f"{len(tokens)} of {cfg.T} tokens evenly spaced")
                      + f" ({len(tokens) * cfg.k} routed rows, all experts, full weights), fp64 numpy, {dt:.1f} s",
            "seconds": round(dt, 2),
            "gpu_vs_oracle_max_rel_err": round(float(diff.max() / np.abs(ref).max()), 5),
            "gpu_vs_oracle_max_err_over_max_abs_rms": round(float((diff / np.maximum(np.abs(ref), rms)).max()), 5)}


if __name__ == "__main__":
    sys.exit(main())
