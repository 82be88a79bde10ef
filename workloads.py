"""Seeded synthetic inputs for the MoE-layer hot path.

This module only *draws* numbers: token rows, expert weights, gate logits and
source-segment boundaries.  It holds none of the layer's arithmetic (no
routing, no permutation, no FFN), so that the CPU oracle and the HIP path can
both be fed from it without sharing any code of the method itself.

Everything is produced by numpy's counter-based Philox generator keyed by
(config seed, tensor id, chunk id); chunks are independent, so large tensors
are drawn by a small thread pool and are bit-identical for any pool size.

bf16 tensors are returned as ``uint16`` arrays holding the bf16 bit patterns
(round-to-nearest-even of the fp32 draw); ``bf16_to_f32`` widens them back.

The five workload shapes follow the expert shapes of the paper's Table 2
(Mixtral-8x7B: N=4096, K=14336, E=8, topk=2; Phi-3.5-MoE: N=4096, K=6400,
E=16, topk=2) plus a tiny test size, a many-small-experts shape and a skewed
load in the spirit of the token-distribution study of Section 5.4; the paper
measures on synthetic token streams of those shapes, not on a dataset.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field, replace
from typing import Dict, Optional

import numpy as np
from numpy.random import Generator, Philox

ACT_GELU = 0
ACT_SWIGLU = 1
ACT_IDENTITY = 2  # test-only: makes the layer linear

_CHUNK = 1 << 22
_TENSOR_X, _TENSOR_W1, _TENSOR_W2, _TENSOR_LOGITS, _TENSOR_SEG = 1, 2, 3, 4, 5


@dataclass(frozen=True)
class MoEConfig:
    name: str
    T: int            # tokens in the receive buffer (paper's M)
    H: int            # token embedding size (paper's N)
    F: int            # expert hidden size (paper's K)
    E: int            # experts
    k: int            # experts per token (paper's topk)
    act: int          # ACT_GELU / ACT_SWIGLU
    S: int            # source segments of the receive buffer
    seed: int
    skew_zipf: float = 0.0        # >0: add log((e+1)^-s / Z) to the logits
    dirichlet_segments: bool = False
    load_std: float = 0.0         # >0: expert popularity with this standard deviation of the per-expert fractions

    @property
    def R(self) -> int:
        return self.T * self.k

    @property
    def F1(self) -> int:
        """Columns of W1: gate|up for SwiGLU, F otherwise."""
        return 2 * self.F if self.act == ACT_SWIGLU else self.F

    @property
    def flops(self) -> float:
        return 2.0 * self.R * self.H * self.F1 + 2.0 * self.R * self.F * self.H


CONFIGS: Dict[str, MoEConfig] = {
    "tiny": MoEConfig("tiny", T=128, H=256, F=512, E=4, k=2, act=ACT_GELU, S=8, seed=0),
    "mixtral": MoEConfig("mixtral", T=8192, H=4096, F=14336, E=8, k=2, act=ACT_SWIGLU, S=8, seed=1),
    "qwen2": MoEConfig("qwen2", T=4096, H=3584, F=2560, E=64, k=8, act=ACT_SWIGLU, S=8, seed=2),
    "phi35": MoEConfig("phi35", T=16384, H=4096, F=6400, E=16, k=2, act=ACT_SWIGLU, S=8, seed=3),
    "skewed": MoEConfig("skewed", T=32768, H=4096, F=14336, E=8, k=2, act=ACT_SWIGLU, S=8, seed=4,
                        skew_zipf=1.2, dirichlet_segments=True),
}


# Further shapes of the paper's evaluation, for the rows marked "next": Table 2's Qwen2-MoE-2.7B row, the
# tensor-parallel slices of the Mixtral expert (Fig. 12: F/TP columns per GPU) and the token-distribution study
# of Fig. 14 (std of the per-expert load fractions; 0.032 is the production average the paper quotes).
CONFIGS.update({
    "qwen2_table2": MoEConfig("qwen2_table2", T=8192, H=2048, F=1408, E=64, k=4, act=ACT_SWIGLU, S=8, seed=5),
    "mixtral_tp2": MoEConfig("mixtral_tp2", T=8192, H=4096, F=7168, E=8, k=2, act=ACT_SWIGLU, S=8, seed=6),
    "mixtral_tp4": MoEConfig("mixtral_tp4", T=8192, H=4096, F=3584, E=8, k=2, act=ACT_SWIGLU, S=8, seed=7),
    "mixtral_tp8": MoEConfig("mixtral_tp8", T=8192, H=4096, F=1792, E=8, k=2, act=ACT_SWIGLU, S=8, seed=8),
    "mixtral_std032": MoEConfig("mixtral_std032", T=8192, H=4096, F=14336, E=8, k=2, act=ACT_SWIGLU, S=8, seed=9,
                                load_std=0.032),
    "mixtral_std05": MoEConfig("mixtral_std05", T=8192, H=4096, F=14336, E=8, k=2, act=ACT_SWIGLU, S=8, seed=10,
                               load_std=0.05),
})


def f32_to_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest even.  Finite inputs only."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> fp32, exact."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_chunk(seed: int, tensor: int, chunk: int, n: int) -> np.ndarray:
    g = Generator(Philox(key=[(seed << 8) | tensor, chunk]))
    return g.standard_normal(n, dtype=np.float32)


def _fill_normal(out_f32: Optional[np.ndarray], out_bf16: Optional[np.ndarray], seed: int, tensor: int,
                 scale: float, threads: int) -> None:
    n = (out_f32 if out_f32 is not None else out_bf16).size
    flat32 = out_f32.reshape(-1) if out_f32 is not None else None
    flat16 = out_bf16.reshape(-1) if out_bf16 is not None else None

    def work(c: int) -> None:
        lo = c * _CHUNK
        hi = min(n, lo + _CHUNK)
        v = _normal_chunk(seed, tensor, c, hi - lo)
        if scale != 1.0:
            v *= np.float32(scale)
        if flat32 is not None:
            flat32[lo:hi] = v
        if flat16 is not None:
            flat16[lo:hi] = f32_to_bf16(v)

    nchunks = (n + _CHUNK - 1) // _CHUNK
    if threads <= 1 or nchunks == 1:
        for c in range(nchunks):
            work(c)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, range(nchunks)))


def normal_bf16(shape, seed: int, tensor: int, std: float = 1.0, threads: int = 8) -> np.ndarray:
    out = np.empty(shape, dtype=np.uint16)
    _fill_normal(None, out, seed, tensor, std, threads)
    return out


def normal_f32(shape, seed: int, tensor: int, std: float = 1.0, threads: int = 8) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    _fill_normal(out, None, seed, tensor, std, threads)
    return out


def segment_offsets(cfg: MoEConfig) -> np.ndarray:
    """Boundaries [S+1] of the per-source segments of the receive buffer.

    Equal split by default; for the skewed workload the sizes are a
    Dirichlet(1) draw times T, rounded by largest remainder (a segment may be
    empty)."""
    T, S = cfg.T, cfg.S
    if not cfg.dirichlet_segments:
        base, rem = divmod(T, S)
        sizes = np.full(S, base, dtype=np.int64)
        sizes[:rem] += 1
    else:
        g = Generator(Philox(key=[(cfg.seed << 8) | _TENSOR_SEG, 0]))
        p = g.dirichlet(np.ones(S))
        raw = p * T
        sizes = np.floor(raw).astype(np.int64)
        short = T - int(sizes.sum())
        order = np.argsort(-(raw - sizes), kind="stable")
        sizes[order[:short]] += 1
    off = np.zeros(S + 1, dtype=np.int32)
    off[1:] = np.cumsum(sizes)
    assert off[-1] == T
    return off


def gate_logits(cfg: MoEConfig, threads: int = 8) -> np.ndarray:
    """fp32 gate logits [T,E] ~ N(0,1), plus the per-expert popularity bias of the skewed workload."""
    g = normal_f32((cfg.T, cfg.E), cfg.seed, _TENSOR_LOGITS, 1.0, threads)
    if cfg.skew_zipf > 0.0:
        pop = np.arange(1, cfg.E + 1, dtype=np.float64) ** (-cfg.skew_zipf)
        pop /= pop.sum()
        g += np.log(pop).astype(np.float32)[None, :]
    if cfg.load_std > 0.0:
        # per-expert bias that spreads the popularity linearly around 1/E.  Top-2 routing over 8 experts amplifies
        # the spread of the bias by about 1/0.78 (measured), hence the factor: the realised standard deviation of
        # the per-expert load fractions then lands within a few percent of load_std
        ramp = np.linspace(-1.0, 1.0, cfg.E)
        frac = 1.0 / cfg.E + 0.78 * cfg.load_std * ramp / ramp.std()
        frac = np.clip(frac, 1e-3, None)
        g += np.log(frac / frac.sum()).astype(np.float32)[None, :]
    return g


@dataclass
class MoEInputs:
    cfg: MoEConfig
    x: np.ndarray          # uint16 bf16 bits [T,H]
    W1: np.ndarray         # uint16 bf16 bits [E,H,F1]  (SwiGLU: columns [0,F) gate, [F,2F) up)
    W2: np.ndarray         # uint16 bf16 bits [E,F,H]
    logits: np.ndarray     # fp32 [T,E]
    seg_offsets: np.ndarray  # int32 [S+1]


def make_inputs(cfg: MoEConfig, threads: int = 8, weights: bool = True) -> MoEInputs:
    """Draw every input tensor of one workload.  Weight std is 1/sqrt(fan_in)."""
    x = normal_bf16((cfg.T, cfg.H), cfg.seed, _TENSOR_X, 1.0, threads)
    if weights:
        W1 = normal_bf16((cfg.E, cfg.H, cfg.F1), cfg.seed, _TENSOR_W1, 1.0 / math.sqrt(cfg.H), threads)
        W2 = normal_bf16((cfg.E, cfg.F, cfg.H), cfg.seed, _TENSOR_W2, 1.0 / math.sqrt(cfg.F), threads)
    else:
        W1 = np.empty((0,), np.uint16)
        W2 = np.empty((0,), np.uint16)
    return MoEInputs(cfg, x, W1, W2, gate_logits(cfg, threads), segment_offsets(cfg))


def scaled(cfg: MoEConfig, **kw) -> MoEConfig:
    """A copy of a workload with some fields replaced (used for reduced-size parity cases)."""
    return replace(cfg, **kw)
