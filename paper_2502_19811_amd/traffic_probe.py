"""What each kind of data movement of a GroupGEMM K step costs at the board's power limit.

Runs the library's probe kernels (moe_probe_mfma, moe_probe_mix): the register-only MFMA loop the GroupGEMM is built
from, then the same loop with LDS fragment reads, global->LDS loads (L2-resident or with a quarter of them streaming
from HBM) and a workgroup barrier added at the rates of the 256 x 256 tile.  Every line is a power-limited rate: the
matrix pipes are busy all the time, so TFLOP/s follows the clock the board can hold with that mix.

    python -m paper_2502_19811_amd.traffic_probe
"""
from __future__ import annotations

import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def main() -> int:
    import torch

    import paper_2502_19811_amd as moe

    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    scratch = torch.randint(0, 255, ((n_cu + 1) * (4 << 20),), dtype=torch.uint8, device="cuda")
    # random bytes are not all finite bf16 values: overwrite with a small-valued bf16 pattern
    scratch.view(torch.bfloat16).copy_(torch.rand(scratch.numel() // 2, device="cuda", dtype=torch.float32).sub_(0.5)
                                       .to(torch.bfloat16))
    iters = 200000   # K steps (32 x 32768 flop per wavefront each)
    mix = lambda mode: (lambda: moe.moe_probe_mix(mode, iters, scratch, with_clock=True))
    rows = [("MFMA loop, zeros", lambda: (moe.moe_probe_mfma(False, iters // 2, scratch), None)),
            ("MFMA loop, random bf16", lambda: (moe.moe_probe_mfma(True, iters // 2, scratch), None)),
            ("mix 0: MFMA only (random bf16 from LDS)", mix(0)),
            ("mix 1: + LDS fragment reads", mix(1)),
            ("mix 3: + global->LDS loads, L2-resident", mix(3)),
            ("mix 7: + workgroup barrier per K step", mix(7)),
            ("mix 11: loads with a quarter from HBM, no barrier", mix(11)),
            ("mix 15: everything", mix(15)),
            ("MFMA loop, random bf16 (again)", lambda: (moe.moe_probe_mfma(True, iters // 2, scratch), None)),
            ("16x16x32 MFMA loop, random bf16", lambda: (moe.moe_probe_mfma(2, iters // 2, scratch), None)),
            ("16x16x32 mix 16: MFMA only", mix(16)),
            ("16x16x32 mix 17: + LDS fragment reads", mix(17)),
            ("16x16x32 mix 23: + loads from the L2 and barrier", mix(23)),
            ("16x16x32 mix 31: everything", mix(31))]
    print("| loop | TFLOP/s | of the random-data MFMA loop | core clock GHz | matrix cores busy |")
    print("|---|---|---|---|---|")
    base = None
    for name, fn in rows:
        v, ghz = fn()
        if name.startswith("MFMA loop, random") and base is None:
            base = v
        rel = f"{v / base:.3f}" if base else ""
        # a SIMD issues one 32x32x16 MFMA (32768 flop) per 32 cycles: 1024 flop per cycle
        busy = f"{v * 1e12 / (n_cu * 4 * ghz * 1e9 * 1024):.2f}" if ghz else ""
        print(f"| {name} | {v:.0f} | {rel} | {ghz:.2f} | {busy} |" if ghz else f"| {name} | {v:.0f} | {rel} | | |", flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
