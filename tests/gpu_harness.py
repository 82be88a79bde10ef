"""Helpers for the GPU parity tests: upload one workload, run the HIP path through the C ABI, fetch results."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np
import torch

import paper_2502_19811_amd as moe
import workloads as wl

# max relative error the layer output may have against the fp64 oracle (bf16 inputs, fp32 accumulation)
REL_TOL = 2e-2


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def bf16_to_np(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy().astype(np.float64)


@dataclass
class GpuRun:
    out: np.ndarray                 # fp64 view of the bf16 output [T,H]
    counts: np.ndarray
    offsets: np.ndarray
    perm: np.ndarray
    inv_perm: np.ndarray
    tiles: Dict[str, np.ndarray]
    status: int


class GpuLayer:
    """One plan + resident inputs; forward() can be called repeatedly."""

    def __init__(self, cfg: wl.MoEConfig, inp: wl.MoEInputs, ids: np.ndarray, w: np.ndarray,
                 options: Optional[Dict[str, int]] = None, packed: bool = False):
        """packed: the weights are re-laid out once with moe_pack_weights and the forwards take the packed buffers."""
        self.cfg = cfg
        self.plan = moe.moe_plan_create(cfg.T, cfg.H, cfg.F, cfg.E, cfg.k, cfg.S, cfg.act, inp.seg_offsets.tolist())
        for key, val in (options or {}).items():
            moe.moe_plan_set_option(self.plan, key, val)
        self.x = dev_bf16(inp.x)
        self.W1 = dev_bf16(inp.W1) if inp.W1.size else torch.zeros(8, dtype=torch.bfloat16, device="cuda")
        self.W2 = dev_bf16(inp.W2) if inp.W2.size else torch.zeros(8, dtype=torch.bfloat16, device="cuda")
        if packed and inp.W1.size:
            W1p, W2p = torch.empty_like(self.W1), torch.empty_like(self.W2)
            moe.moe_pack_weights(self.plan, self.W1, self.W2, W1p, W2p)
            torch.cuda.synchronize()
            self.W1, self.W2 = W1p, W2p          # the plain copies are dropped: a forward must not need them
            moe.moe_plan_set_option(self.plan, "weights_packed", 1)
        self.ids = torch.from_numpy(ids).cuda()
        self.w = torch.from_numpy(w).cuda()
        self.out = torch.zeros((cfg.T, cfg.H), dtype=torch.bfloat16, device="cuda")
        self.ws = torch.zeros(max(moe.moe_plan_workspace_bytes(self.plan), 256), dtype=torch.uint8, device="cuda")

    def forward(self, seg_ready=None, epoch: int = 0, stream=None):
        moe.moe_layer_forward(self.plan, self.x, self.ids, self.w, self.W1, self.W2, self.cfg.act, self.out, self.ws,
                              seg_ready, epoch, stream)

    def results(self) -> GpuRun:
        cfg = self.cfg
        i32 = dict(dtype=torch.int32, device="cuda")
        counts = torch.zeros(cfg.E, **i32)
        offsets = torch.zeros(cfg.E + 1, **i32)
        perm = torch.zeros(max(cfg.R, 1), **i32)
        inv = torch.zeros(max(cfg.R, 1), **i32)
        mt = max(moe.moe_plan_max_tiles(self.plan), 1)
        n_tiles = torch.zeros(1, **i32)
        te, tr0, tr, ts, th = (torch.zeros(mt, **i32) for _ in range(5))
        if cfg.T > 0:
            moe.moe_get_index_outputs(self.plan, self.ws, counts, offsets, perm, inv)
            moe.moe_get_tile_table(self.plan, self.ws, n_tiles, te, tr0, tr, ts, th)
        status = moe.moe_last_device_status(self.plan, self.ws) if cfg.T > 0 else 0
        torch.cuda.synchronize()
        n = int(n_tiles.item())
        tiles = {"expert": te[:n].cpu().numpy(), "row0": tr0[:n].cpu().numpy(), "rows": tr[:n].cpu().numpy(),
                 "ready_seg": ts[:n].cpu().numpy(), "height": th[:n].cpu().numpy()}
        return GpuRun(bf16_to_np(self.out), counts.cpu().numpy(), offsets.cpu().numpy(), perm[:cfg.R].cpu().numpy(),
                      inv[:cfg.R].cpu().numpy(), tiles, status)

    def close(self):
        moe.moe_plan_destroy(self.plan)
        self.plan = None


def error_metrics(got: np.ndarray, ref: np.ndarray):
    """(max|g-r| / max|r|,  max_i |g_i-r_i| / max(|r_i|, rms(r))): both must stay below REL_TOL."""
    diff = np.abs(got - ref)
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 1.0
    a = float(diff.max() / max(np.abs(ref).max(), 1e-30)) if ref.size else 0.0
    b = float((diff / np.maximum(np.abs(ref), rms)).max()) if ref.size else 0.0
    return a, b
