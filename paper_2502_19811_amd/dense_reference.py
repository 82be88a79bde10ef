"""Context measurement, no part of the library: the vendor's dense bf16 GEMM (torch.matmul, i.e. hipBLASLt) on the
two GEMM shapes of the Mixtral-shaped layer, with the weight operand stored as the layer takes it (K x N row-major)
and transposed (N x K), on random data of the workload's scale.  Printed next to the library's own register-only
MFMA loop on the same board, which is what both have to be read against.

    python -m paper_2502_19811_amd.dense_reference
"""
from __future__ import annotations

import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def main() -> int:
    import torch

    import paper_2502_19811_amd as moe

    torch.manual_seed(0)
    scratch = torch.zeros(1 << 22, dtype=torch.uint8, device="cuda")
    print(f"MFMA loop, random bf16: {moe.moe_probe_mfma(True, 100000, scratch):.0f} TFLOP/s", flush=True)
    print("| M x K x N | weight layout | us | TFLOP/s |")
    print("|---|---|---|---|")
    for M, K, N in ((16384, 4096, 28672), (16384, 14336, 4096)):
        a = torch.randn(M, K, device="cuda", dtype=torch.bfloat16)
        b = (torch.randn(K, N, device="cuda", dtype=torch.float32) / K ** 0.5).to(torch.bfloat16)
        bt = b.t().contiguous()
        for name, f in (("K x N (as the layer's weights)", lambda: a @ b), ("N x K (transposed copy)", lambda: a @ bt.t())):
            for _ in range(5):
                f()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                f()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 20
            print(f"| {M} x {K} x {N} | {name} | {ms * 1e3:.0f} | {2.0 * M * K * N / ms / 1e9:.0f} |", flush=True)
        del a, b, bt
    print(f"MFMA loop, random bf16 (again): {moe.moe_probe_mfma(True, 100000, scratch):.0f} TFLOP/s", flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
