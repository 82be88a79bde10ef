"""Pins for the oracle's routing, row order, tile readiness and buffer sizes (CPU only)."""
import numpy as np
import pytest
from scipy.special import softmax

import workloads as wl
from oracle import moe_oracle as orc
from conftest import read_golden


# ---------------------------------------------------------------- routing
def _rand_logits(T, E, seed):
    return wl.normal_f32((T, E), seed, 40, 1.0, threads=1)


@pytest.mark.parametrize("T,E,k", [(64, 4, 2), (33, 64, 8), (17, 8, 8), (5, 16, 1)])
def test_route_weights_closed_forms(T, E, k):
    g = _rand_logits(T, E, 7)
    ids, w = orc.route_topk(g, k)
    assert ids.dtype == np.int32 and w.dtype == np.float32 and ids.shape == (T, k)
    # renormalised weights sum to one
    np.testing.assert_allclose(w.sum(axis=1, dtype=np.float64), 1.0, atol=1e-6)
    # softmax-then-renormalise over the kept k equals a softmax over the kept logits alone
    kept = np.take_along_axis(g.astype(np.float64), ids.astype(np.int64), axis=1)
    np.testing.assert_allclose(w, softmax(kept, axis=1), atol=1e-7)
    # descending probability per slot, distinct experts, in range
    assert (np.diff(w.astype(np.float64), axis=1) <= 1e-9).all()
    assert all(len(set(r)) == k for r in ids.tolist())
    assert ids.min() >= 0 and ids.max() < E


def test_route_k_equals_E_is_full_softmax():
    g = _rand_logits(9, 8, 3)
    ids, w = orc.route_topk(g, 8)
    full = softmax(g.astype(np.float64), axis=1)
    np.testing.assert_allclose(w, np.take_along_axis(full, ids.astype(np.int64), axis=1), atol=1e-7)


def test_route_bruteforce_selection():
    g = _rand_logits(50, 16, 11)
    ids, _ = orc.route_topk(g, 4)
    for t in range(g.shape[0]):
        left = list(range(16))
        chosen = []
        for _ in range(4):
            best = left[0]
            for e in left[1:]:
                if g[t, e] > g[t, best]:      # strict: equal values keep the lower id
                    best = e
            chosen.append(best)
            left.remove(best)
        assert chosen == ids[t].tolist()


def test_route_ties_go_to_lower_expert():
    g = np.array([[1.0, 1.0, 0.0, 1.0], [0.0, 0.0, 0.0, 0.0], [-1.0, 3.0, 3.0, -1.0]], np.float32)
    ids, w = orc.route_topk(g, 2)
    assert ids.tolist() == [[0, 1], [0, 1], [1, 2]]
    np.testing.assert_allclose(w, 0.5)


def test_route_ties_among_many_experts():
    """Rows long enough that a sort which is not stable reorders equal logits (short rows hide that)."""
    rng = np.random.default_rng(5)
    E, k = 64, 8
    g = rng.integers(0, 3, size=(200, E)).astype(np.float32)      # three distinct values: ties everywhere
    ids, _ = orc.route_topk(g, k)
    for t in range(g.shape[0]):
        want = sorted(range(E), key=lambda e: (-float(g[t, e]), e))[:k]
        assert ids[t].tolist() == want


def test_route_fig2_example():
    for row in read_golden("routing_fig2.txt"):
        bar = row.index("|")
        logits = np.array([[float(v) for v in row[:bar]]], np.float32)
        want = [int(v) for v in row[bar + 1:]]
        ids, _ = orc.route_topk(logits, len(want))
        assert ids[0].tolist() == want


# ---------------------------------------------------------------- permutation
def _rand_ids(T, E, k, seed):
    ids, _ = orc.route_topk(_rand_logits(T, E, seed), k)
    return ids


@pytest.mark.parametrize("T,E,k", [(128, 4, 2), (300, 64, 8), (77, 8, 3), (1, 4, 2), (40, 16, 1)])
def test_permutation_vs_python_sorted_and_invariants(T, E, k):
    ids = _rand_ids(T, E, k, 5)
    counts, offsets, perm, inv = orc.build_permutation(ids, E)
    R = T * k
    flat = ids.reshape(-1).tolist()
    assert perm.tolist() == sorted(range(R), key=flat.__getitem__)      # Python's sort is stable
    assert sorted(perm.tolist()) == list(range(R))                       # bijection on the (token, slot) pairs
    assert (inv[perm] == np.arange(R)).all() and (perm[inv] == np.arange(R)).all()
    assert int(counts.sum()) == R and offsets[0] == 0 and offsets[-1] == R
    assert counts.tolist() == [flat.count(e) for e in range(E)]
    keys = np.array(flat)[perm]
    assert (np.diff(keys) >= 0).all()
    for e in range(E):
        seg = perm[offsets[e]:offsets[e + 1]]
        assert (keys[offsets[e]:offsets[e + 1]] == e).all()
        assert (np.diff(seg) > 0).all()                                  # ascending pair id = source order


def test_permutation_empty_experts():
    ids = np.array([[2, 5], [5, 2], [2, 5]], np.int32)
    counts, offsets, perm, inv = orc.build_permutation(ids, 8)
    assert counts.tolist() == [0, 0, 3, 0, 0, 3, 0, 0]
    assert perm.tolist() == [0, 3, 4, 1, 2, 5]
    assert inv.tolist() == [0, 3, 4, 1, 2, 5]


def test_uniform_load_count_section_5_4():
    (M, topk, E, rows), = [[int(v) for v in r] for r in read_golden("uniform_load.txt")]
    t = np.arange(M)[:, None]
    ids = ((t * topk + np.arange(topk)[None, :]) % E).astype(np.int32)   # perfectly uniform routing
    counts, offsets, perm, _ = orc.build_permutation(ids, E)
    assert counts.tolist() == [rows] * E
    assert perm.size == orc.shared_tensor_shape(M, topk, 4096)[0] == M * topk


def test_table3_buffer_sizes():
    for M, N, mb in [[int(v) for v in r] for r in read_golden("table3_buffer_mb.txt")]:
        assert orc.receive_buffer_bytes(M, N) == mb << 20


# ---------------------------------------------------------------- readiness of groups of rows
def test_rows_ready_segment_is_the_segment_of_the_last_row():
    """Rows of an expert are in source order (Fig. 5), so the latest segment of any run of an expert's rows is the
    segment of its last row; checked by brute force over every run of a few lengths."""
    cfg = wl.scaled(wl.CONFIGS["skewed"], T=700, E=8, k=2)
    seg = wl.segment_offsets(cfg)
    ids = _rand_ids(cfg.T, cfg.E, cfg.k, 9)
    _, offsets, perm, _ = orc.build_permutation(ids, cfg.E)

    def seg_of(t):
        return next(j for j in range(cfg.S) if seg[j] <= t < seg[j + 1])

    for e in range(cfg.E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        for n in (1, 7, 64):
            for a in range(lo, max(lo, hi - n + 1), 13):
                segs = [seg_of(int(perm[r]) // cfg.k) for r in range(a, a + n)]
                assert segs == sorted(segs)
                assert orc.rows_ready_segment(seg, perm, cfg.k, a, n) == max(segs) == segs[-1]
    # across experts the order restarts: a run spanning two experts needs the maximum, not the last row
    a = int(offsets[1]) - 3
    segs = [seg_of(int(perm[r]) // cfg.k) for r in range(a, a + 6)]
    assert orc.rows_ready_segment(seg, perm, cfg.k, a, 6) == max(segs)


def test_segment_offsets_properties():
    for cfg in wl.CONFIGS.values():
        so = wl.segment_offsets(cfg)
        assert so[0] == 0 and so[-1] == cfg.T and (np.diff(so) >= 0).all() and so.size == cfg.S + 1
    eq = wl.segment_offsets(wl.CONFIGS["mixtral"])
    assert (np.diff(eq) == 1024).all()
