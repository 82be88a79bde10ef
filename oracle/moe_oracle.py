"""CPU oracle for the single-GPU hot path of the MoE layer.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path may import this module: it exists so that the HIP
kernels can be checked against a plain, slow, obviously correct statement of
what the layer computes.  It shares no code with the HIP path (no kernels,
headers, helpers or tables); both are fed by the seeded generators of
``workloads.py``.

What is computed (paper Section 2.1: a gate picks ``topk`` experts per token,
the token goes through the two feed-forward GEMMs of each chosen expert, and
the ``topk`` results are reduced back into one row per token; Section 3.1 and
Fig. 4: both pipelines meet in a shared tensor of ``M*topk`` rows; Section
3.1.2 and Fig. 5: inside an expert the rows are ordered by source rank).

All floating point work is fp64 over the exact values of the bf16 inputs.  The
one deliberate rounding is the activation output ``h``, which the method keeps
in a bf16 buffer between the two GEMMs (Section 5.5 names BF16/FP16 as the
buffer types); ``round_h=False`` switches it off.

Pins (see tests/test_oracle_*.py): routing against closed forms and a library
softmax; the permutation against Python's stable ``sorted`` and the bijection /
count invariants (uniform load M*topk/E = 2048 rows of Section 5.4); the FFN
and combine against a per-token brute-force loop that uses no permutation, a
dense two-layer MLP evaluated with torch CPU, linear-layer and equal-weight
special cases; the activations against printed constants and torch; the
buffer size against Table 3.  The absolute output values of the layer are not
printed anywhere in the paper: for those, parity is pinned only through the
reductions above.
"""
from __future__ import annotations

from typing import Optional, Sequence, Tuple

import numpy as np
from scipy.special import erf

ACT_GELU = 0
ACT_SWIGLU = 1
ACT_IDENTITY = 2


# --------------------------------------------------------------------------
# bf16 <-> fp64
# --------------------------------------------------------------------------
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact value of bf16 bit patterns (uint16) as fp64."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def round_f64_to_bf16(v: np.ndarray) -> np.ndarray:
    """Round fp64 to the nearest bf16 value (ties to even), returned as fp64.

    bf16 keeps 7 explicit mantissa bits, fp64 has 52: the low 45 bits are
    rounded away directly in the fp64 bit pattern, so there is no double
    rounding through fp32.  Valid for finite values inside bf16's normal
    range, which is all the layer produces."""
    u = np.ascontiguousarray(v, dtype=np.float64).view(np.uint64)
    drop = np.uint64(45)
    lsb = (u >> drop) & np.uint64(1)
    r = (u + (np.uint64((1 << 44) - 1) + lsb)) & ~np.uint64((1 << 45) - 1)
    return r.view(np.float64)


def f64_to_bf16_bits(v: np.ndarray) -> np.ndarray:
    r = round_f64_to_bf16(v).astype(np.float32)  # exact: 8 significant bits
    return (r.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


# --------------------------------------------------------------------------
# A1. Routing (Section 2.1: a gate network selects the topk experts per token)
# --------------------------------------------------------------------------
def route_topk(logits: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """softmax over all E experts -> the k most probable -> renormalise over the kept k.

    Slot 0 is the most probable expert; equal logits go to the lower expert id.
    The choice is made on the logits themselves (softmax is monotonic), so no
    rounding can change it.  Returns ids int32 [T,k] and weights fp32 [T,k]."""
    g = np.asarray(logits)
    T, E = g.shape
    assert 1 <= k <= E
    # stable argsort of -logit: descending value, ties by ascending expert id
    order = np.argsort(-g.astype(np.float64), axis=1, kind="stable")
    ids = order[:, :k].astype(np.int32)
    g64 = g.astype(np.float64)
    p = np.exp(g64 - g64.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    kept = np.take_along_axis(p, ids.astype(np.int64), axis=1)
    w = kept / kept.sum(axis=1, keepdims=True)
    return ids, w.astype(np.float32)


# --------------------------------------------------------------------------
# A4. Shared-tensor row order (Section 3.1.2, Fig. 5)
# --------------------------------------------------------------------------
def build_permutation(topk_ids: np.ndarray, E: int):
    """Row order of the shared tensor.

    Pair id q = t*k + j.  Rows are grouped by expert; inside an expert they are
    in ascending q.  Because source segment s owns the contiguous token range
    [seg_offsets[s], seg_offsets[s+1]), ascending q is also "sorted by source
    rank, local rank first", whatever the segment boundaries are.

    Returns counts[E], offsets[E+1], perm[R] (sorted position -> pair id) and
    inv_perm[R] (pair id -> sorted position), all int32."""
    ids = np.asarray(topk_ids, dtype=np.int64).reshape(-1)
    assert ids.size == 0 or (ids.min() >= 0 and ids.max() < E)
    counts = np.bincount(ids, minlength=E).astype(np.int32)
    offsets = np.zeros(E + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    perm = np.argsort(ids, kind="stable").astype(np.int32)
    inv_perm = np.empty_like(perm)
    inv_perm[perm] = np.arange(perm.size, dtype=np.int32)
    return counts, offsets, perm, inv_perm


def segment_of_token(seg_offsets: np.ndarray, t: np.ndarray) -> np.ndarray:
    """Index s of the source segment with seg_offsets[s] <= t < seg_offsets[s+1] (empty segments skipped)."""
    so = np.asarray(seg_offsets, dtype=np.int64)
    return (np.searchsorted(so, np.asarray(t, dtype=np.int64), side="right") - 1).astype(np.int32)


def rows_ready_segment(seg_offsets: np.ndarray, perm: np.ndarray, k: int, row0: int, nrows: int) -> int:
    """Source segment a group of shared-tensor rows [row0, row0+nrows) has to wait for.

    A GEMM tile cannot start before every token it needs has arrived (Section 2.2.1); segments arrive as wholes,
    so the group is complete when the latest segment any of its rows comes from is there: the maximum over the
    rows.  How rows are cut into tiles is a tuning choice of an implementation and no part of this oracle."""
    toks = np.asarray(perm[row0:row0 + nrows], dtype=np.int64) // k
    return int(segment_of_token(seg_offsets, toks).max())


# --------------------------------------------------------------------------
# A6. Activation between the two GEMMs (not named by the paper; fixed by the workloads)
# --------------------------------------------------------------------------
def activation(G: np.ndarray, act: int) -> np.ndarray:
    """GELU: 0.5*g*(1+erf(g/sqrt 2)).  SwiGLU on [gate | up]: silu(gate)*up with silu(g) = g/(1+exp(-g))."""
    if act == ACT_GELU:
        return 0.5 * G * (1.0 + erf(G / np.sqrt(2.0)))
    if act == ACT_SWIGLU:
        F = G.shape[-1] // 2
        gate, up = G[..., :F], G[..., F:]
        return gate / (1.0 + np.exp(-gate)) * up
    if act == ACT_IDENTITY:
        return G
    raise ValueError(f"unknown activation {act}")


# --------------------------------------------------------------------------
# A5 + A8 + A9. Expert FFN over the shared tensor, then the top-k reduction
# --------------------------------------------------------------------------
def expert_ffn(x_bits, W1_bits, W2_bits, offsets, perm, k: int, act: int, round_h: bool = True,
               col_chunk: int = 4096) -> np.ndarray:
    """Y[p,:] = act(x[perm[p] // k, :] @ W1[e]) @ W2[e] for every sorted row p of expert e, fp64 [R,H]."""
    E = W1_bits.shape[0]
    H = x_bits.shape[1]
    R = perm.size
    Y = np.zeros((R, H), dtype=np.float64)
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi == lo:
            continue
        A = bf16_bits_to_f64(x_bits[perm[lo:hi] // k])
        F1 = W1_bits.shape[2]
        G = np.empty((hi - lo, F1), dtype=np.float64)
        for c in range(0, F1, col_chunk):
            G[:, c:c + col_chunk] = A @ bf16_bits_to_f64(W1_bits[e, :, c:c + col_chunk])
        h = activation(G, act)
        if round_h:
            h = round_f64_to_bf16(h)
        F = h.shape[1]
        acc = np.zeros((hi - lo, H), dtype=np.float64)
        for c in range(0, F, col_chunk):
            acc += h[:, c:c + col_chunk] @ bf16_bits_to_f64(W2_bits[e, c:c + col_chunk, :])
        Y[lo:hi] = acc
    return Y


def combine(Y: np.ndarray, inv_perm: np.ndarray, topk_weights: np.ndarray) -> np.ndarray:
    """out[t,:] = sum_j w[t,j] * Y[inv_perm[t*k+j], :], added in ascending j, fp64 [T,H]."""
    T, k = topk_weights.shape
    w = np.asarray(topk_weights, dtype=np.float64)
    out = np.zeros((T, Y.shape[1]), dtype=np.float64)
    for j in range(k):
        out += w[:, j:j + 1] * Y[inv_perm[np.arange(T) * k + j]]
    return out


def moe_layer(x_bits, W1_bits, W2_bits, topk_ids, topk_weights, act: int, round_h: bool = True) -> np.ndarray:
    """The whole layer on one GPU's share: permutation -> expert FFN -> combine.  Returns fp64 [T,H] (unrounded)."""
    E = W1_bits.shape[0]
    k = topk_ids.shape[1]
    _, offsets, perm, inv_perm = build_permutation(topk_ids, E)
    Y = expert_ffn(x_bits, W1_bits, W2_bits, offsets, perm, k, act, round_h)
    return combine(Y, inv_perm, topk_weights)


def moe_layer_tokens(tokens: Sequence[int], x_bits, W1_bits, W2_bits, topk_ids, topk_weights, act: int,
                     round_h: bool = True) -> np.ndarray:
    """Output rows of a subset of tokens.

    Tokens are independent of each other along M (Section 3.1.1), so the rows
    of a subset are the layer applied to that subset alone."""
    t = np.asarray(tokens, dtype=np.int64)
    return moe_layer(x_bits[t], W1_bits, W2_bits, topk_ids[t], topk_weights[t], act, round_h)


# --------------------------------------------------------------------------
# Sizes the paper states
# --------------------------------------------------------------------------
def shared_tensor_shape(M: int, topk: int, N: int) -> Tuple[int, int]:
    """Global size of the shared tensor of both layers (Fig. 4)."""
    return (M * topk, N)


def receive_buffer_bytes(M: int, N: int, itemsize: int = 2) -> int:
    """Size of the communication buffer: M*N elements, 2*M*N bytes in bf16/fp16 (Section 5.5, Table 3)."""
    return itemsize * M * N
