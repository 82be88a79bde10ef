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
class ForwardResult:
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

    def results(self) -> ForwardResult:
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
        return ForwardResult(bf16_to_np(self.out), counts.cpu().numpy(), offsets.cpu().numpy(), perm[:cfg.R].cpu().numpy(),
                      inv[:cfg.R].cpu().numpy(), tiles, status)

    def schedule(self, layer: int):
        """(items [n, 8] int32 numpy, queues [(first, count, stride)] * 8) of the last forward's tile schedule."""
        cap = max(moe.moe_plan_schedule_capacity(self.plan, layer), 1)
        items = torch.zeros((cap, 8), dtype=torch.int32, device="cuda")
        queues = moe.moe_get_schedule(self.plan, self.ws, layer, items)
        return items.cpu().numpy(), queues

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


def check_tile_table(tiles, cfg, offsets, perm, seg_offsets, tile_m):
    """The M-tile table of a forward, checked through what any valid table has (the paper fixes no tile size or cut
    rule: the rule is the library's): expert-major; the tiles of an expert partition its row range in order; heights
    are kernel variants no taller than tile_m; a tile is full unless it is the expert's last; the segment it waits
    for is the latest segment of its rows (Section 2.2.1), computed here from the oracle's row order."""
    from oracle import moe_oracle as orc
    ex, r0, nr, rs, ht = (np.asarray(tiles[key], dtype=np.int64) for key in ("expert", "row0", "rows", "ready_seg", "height"))
    assert (np.diff(ex) >= 0).all(), "tile table is not expert-major"
    assert np.isin(ht, (64, 128, 256)).all() and (ht <= tile_m).all()
    assert (nr > 0).all() and (nr <= ht).all()
    row_seg = orc.segment_of_token(seg_offsets, np.asarray(perm, dtype=np.int64) // cfg.k).astype(np.int64)
    pos = 0
    for e in range(cfg.E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        idx = np.nonzero(ex == e)[0]
        if hi == lo:
            assert idx.size == 0, f"expert {e} has no rows but {idx.size} tiles"
            continue
        assert idx.size > 0 and (np.diff(idx) == 1).all() and idx[0] == pos
        pos += idx.size
        assert r0[idx[0]] == lo and r0[idx[-1]] + nr[idx[-1]] == hi
        assert (r0[idx[1:]] == r0[idx[:-1]] + nr[idx[:-1]]).all(), f"tiles of expert {e} leave a gap or overlap"
        assert (nr[idx[:-1]] == ht[idx[:-1]]).all(), "only the last tile of an expert may be ragged"
        # little padding: less than the smallest tile, unless the remainder needed a full-height ragged tile
        pad = int(ht[idx].sum()) - (hi - lo)
        assert 0 <= pad < 64 or ht[idx[-1]] == tile_m
    assert pos == ex.size
    for m in range(ex.size):
        assert rs[m] == row_seg[r0[m]:r0[m] + nr[m]].max(), f"tile {m} waits for the wrong segment"


def check_schedule(items, queues, tiles, n_tiles_n, seg_major=False, panel_major=False, waves=None):
    """Invariants of a tile schedule (Fig. 5 / Fig. 6): the queues list every (M-tile, column tile) pair exactly once,
    every record repeats its M-tile's table row, tall tiles come before short ones inside a queue; seg_major: inside
    a height class of a queue the segment waited for never decreases (rows that arrive early first); panel_major:
    inside a height class of a queue the groups of 4 column panels ascend (all M-tiles finish a group before the
    next one starts); waves = (n_waves, S): the queue is wave-major (wave of a tile = ready_seg * n_waves // S), tall
    before short inside a wave, and the M-tiles of an expert inside a wave sweep the column tiles together."""
    n_tiles = len(tiles["row0"])
    seen = np.zeros((n_tiles, n_tiles_n), dtype=np.int32)
    for first, count, stride in queues:
        if count == 0:
            continue
        q = items[first:first + count * stride:stride]
        assert len(q) == count
        m, n = q[:, 0], q[:, 1]
        assert (m >= 0).all() and (m < n_tiles).all() and (n >= 0).all() and (n < n_tiles_n).all()
        np.add.at(seen, (m, n), 1)
        np.testing.assert_array_equal(q[:, 2], tiles["expert"][m])
        np.testing.assert_array_equal(q[:, 3], tiles["row0"][m])
        np.testing.assert_array_equal(q[:, 4], tiles["rows"][m])
        np.testing.assert_array_equal(64 << q[:, 5], tiles["height"][m])
        np.testing.assert_array_equal(q[:, 6], tiles["ready_seg"][m])
        if waves:
            wave = q[:, 6] * waves[0] // waves[1]
            assert (np.diff(wave) >= 0).all(), "a tile of an earlier wave after one of a later wave"
            for wv in np.unique(wave):
                assert (np.diff(q[wave == wv][:, 5]) <= 0).all(), "a taller tile after a shorter one inside a wave"
        else:
            assert (np.diff(q[:, 5]) <= 0).all(), "a taller tile after a shorter one"
        for kind in (2, 1, 0):
            part = q[q[:, 5] == kind]
            if seg_major:
                assert (np.diff(part[:, 6]) >= 0).all(), "segment order violated"
            if panel_major:
                assert (np.diff(part[:, 1] // 4) >= 0).all(), "column-panel groups out of order"
    assert (seen == 1).all(), f"{int((seen == 0).sum())} items missing, {int((seen > 1).sum())} listed more than once"
