"""GPU parity at the full workload sizes, in the launch configuration bench.py times: index outputs compared in
full; layer outputs compared with the oracle in full on the five benchmark workloads and on at least 1024 sampled
tokens on the further workloads (tokens are independent along M, so the oracle computes a sample on its own)."""
import numpy as np
import pytest

import workloads as wl
from oracle import moe_oracle as orc

pytestmark = pytest.mark.gpu


def _sample_tokens(cfg, offsets, perm, tiles, n_min=1024):
    """Tokens behind the first and last row of every expert and of every M-tile (so every tile height, every expert
    and, rows being in source order, every segment an expert has rows from), topped up with evenly spaced tokens to at
    least n_min.  Every sampled token contributes all of its k slots."""
    rows = set()
    for e in range(cfg.E):
        if offsets[e + 1] > offsets[e]:
            rows.update((int(offsets[e]), int(offsets[e + 1]) - 1))
    for r0, n in zip(tiles["row0"], tiles["rows"]):
        rows.update((int(r0), int(r0 + n - 1)))
    toks = {int(perm[r]) // cfg.k for r in rows}
    so = wl.segment_offsets(cfg)
    for s in range(cfg.S):                      # first and last token of every source segment
        if so[s + 1] > so[s]:
            toks.update((int(so[s]), int(so[s + 1]) - 1))
    n_even = max(n_min - len(toks), 64)
    toks.update(np.linspace(0, cfg.T - 1, n_even).astype(int).tolist())
    extra = 0
    while len(toks) < n_min:                    # evenly spaced picks may coincide with the others
        toks.add((7919 * extra) % cfg.T)
        extra += 1
    return np.array(sorted(toks), dtype=np.int64)


def _run(cfg, inp, ids, w, options=None, packed=False):
    import gpu_harness as H
    layer = H.GpuLayer(cfg, inp, ids, w, options, packed=packed)
    layer.forward()
    run = layer.results()
    layer.close()
    assert run.status == 0
    return run


def _check_index_outputs(run, cfg, ids, inp):
    import gpu_harness as H
    counts, offsets, perm, inv = orc.build_permutation(ids, cfg.E)
    np.testing.assert_array_equal(run.counts, counts)
    np.testing.assert_array_equal(run.offsets, offsets)
    np.testing.assert_array_equal(run.perm, perm)
    np.testing.assert_array_equal(run.inv_perm, inv)
    H.check_tile_table(run.tiles, cfg, offsets, perm, inp.seg_offsets, int(run.tiles["height"].max()))
    return offsets, perm


@pytest.mark.parametrize("name", ["mixtral", "qwen2", "phi35", "skewed"])
def test_full_size_whole_output_against_the_oracle(name):
    """Every output element of the benchmark workloads against the oracle (fp64 on the host: seconds to about a
    minute on the GPU machine's cores), in token chunks so that the oracle's intermediates stay a few GB."""
    import gpu_harness as H
    cfg = wl.CONFIGS[name]
    print(f"whole-output parity {name}: generating inputs", flush=True)
    inp = wl.make_inputs(cfg, threads=16)
    ids, w = orc.route_topk(inp.logits, cfg.k)
    run = _run(cfg, inp, ids, w)
    _check_index_outputs(run, cfg, ids, inp)
    chunk = 16384 if name == "skewed" else cfg.T
    worst = (0.0, 0.0)
    for lo in range(0, cfg.T, chunk):
        toks = np.arange(lo, min(cfg.T, lo + chunk))
        print(f"  oracle on tokens [{lo}, {toks[-1] + 1})", flush=True)
        ref = orc.moe_layer_tokens(toks, inp.x, inp.W1, inp.W2, ids, w, cfg.act)
        a, b = H.error_metrics(run.out[toks], ref)
        print(f"  err {a:.3e} {b:.3e}", flush=True)
        worst = (max(worst[0], a), max(worst[1], b))
    assert worst[0] <= H.REL_TOL and worst[1] <= H.REL_TOL


@pytest.mark.parametrize("name", ["qwen2_table2", "mixtral_tp2", "mixtral_tp4", "mixtral_tp8", "mixtral_std032",
                                  "mixtral_std05"])
def test_full_size_sampled_parity(name):
    """The further workloads (Table 2's Qwen2 row, the tensor-parallel slices of Fig. 12, the load-imbalance study of
    Fig. 14): index outputs in full, layer output on at least 1024 tokens chosen to cover every expert, every M-tile's
    first and last row, every source segment and all k slots."""
    import gpu_harness as H
    cfg = wl.CONFIGS[name]
    print(f"full-size parity {name}: generating inputs", flush=True)
    inp = wl.make_inputs(cfg, threads=16)
    ids, w = orc.route_topk(inp.logits, cfg.k)
    run = _run(cfg, inp, ids, w)
    offsets, perm = _check_index_outputs(run, cfg, ids, inp)
    toks = _sample_tokens(cfg, offsets, perm, run.tiles)
    assert len(toks) >= 1024
    print(f"  oracle on {len(toks)} sampled tokens", flush=True)
    ref = orc.moe_layer_tokens(toks, inp.x, inp.W1, inp.W2, ids, w, cfg.act)
    a, b = H.error_metrics(run.out[toks], ref)
    print(f"  err {a:.3e} {b:.3e}", flush=True)
    assert a <= H.REL_TOL and b <= H.REL_TOL
    # nothing outside the sample is garbage: finite everywhere, and of the sample's magnitude
    assert np.isfinite(run.out).all()
    assert 0.5 < run.out.std() / ref.std() < 2.0


@pytest.mark.parametrize("name", ["mixtral", "qwen2_table2", "qwen2", "skewed"])
def test_full_size_token_reversal_moves_every_row_bit_for_bit(name):
    """Every output row is the same sum in the same order wherever its token sits: reversing the token order reverses
    the output rows exactly.  This checks every row of the full-size output, not a sample, against a run in which
    each routed row lands in a different tile and a different position of it."""
    cfg = wl.CONFIGS[name]
    print(f"token reversal {name}: generating inputs", flush=True)
    inp = wl.make_inputs(cfg, threads=16)
    ids, w = orc.route_topk(inp.logits, cfg.k)
    base = _run(cfg, inp, ids, w)
    rev_seg = (cfg.T - inp.seg_offsets[::-1]).astype(np.int32)       # the segments travel with their tokens
    rev = wl.MoEInputs(cfg, np.ascontiguousarray(inp.x[::-1]), inp.W1, inp.W2, np.ascontiguousarray(inp.logits[::-1]),
                       rev_seg)
    print("  reversed forward", flush=True)
    r2 = _run(cfg, rev, np.ascontiguousarray(ids[::-1]), np.ascontiguousarray(w[::-1]))
    np.testing.assert_array_equal(r2.out[::-1], base.out)


def test_full_size_variants_give_the_same_bits():
    """On the Mixtral-shaped workload, at full size: the in-kernel reduction of finished column panels with and without
    data-movement workgroups (16 panels, 32 token chunks each), the source-ordered layer0 schedule, the packed
    weights, the 128-row tiling and the one-launch variant of the two GroupGEMMs all give the default run's output
    bit for bit."""
    cfg = wl.CONFIGS["mixtral"]
    print("variants mixtral: generating inputs", flush=True)
    inp = wl.make_inputs(cfg, threads=16)
    ids, w = orc.route_topk(inp.logits, cfg.k)
    base = _run(cfg, inp, ids, w)
    for opts, packed in (({"layer1_order": 1, "n_dm": 16}, False), ({"layer1_order": 1, "n_dm": 0}, False),
                         ({"layer0_order": 1}, False), ({}, True), ({"tile_m": 128}, False),
                         ({"fuse_layers": 1, "spin_limit": 1 << 18}, True), ({"layer1_order": 2}, True),
                         ({"n_prefetch": 8}, True), ({"deep_short_tiles": 0}, True)):
        print(f"  options {opts} packed {packed}", flush=True)
        run = _run(cfg, inp, ids, w, opts, packed)
        np.testing.assert_array_equal(run.out, base.out)
        np.testing.assert_array_equal(run.perm, base.perm)


def test_prefetching_workgroups_leave_the_output_unchanged():
    """Table 2's Qwen2 row (64 small experts, the shape the weight prefetch is for): with 8, 16 and 32 of the 256
    workgroups of each GroupGEMM launch prefetching weight panels instead of computing tiles, near and far ahead of
    the queue heads, and with the strided queues of the source-segment order, the output is the default run's bit
    for bit."""
    cfg = wl.CONFIGS["qwen2_table2"]
    print("prefetch qwen2_table2: generating inputs", flush=True)
    inp = wl.make_inputs(cfg, threads=16)
    ids, w = orc.route_topk(inp.logits, cfg.k)
    base = _run(cfg, inp, ids, w, {}, True)
    for opts in ({"n_prefetch": 8}, {"n_prefetch": 16, "prefetch_ahead": 4, "prefetch_behind": 0},
                 {"n_prefetch": 32, "prefetch_ahead": 64, "prefetch_behind": 32}, {"n_prefetch": 8, "layer0_order": 1},
                 {"n_prefetch": 16, "n_cu": 64}, {"n_prefetch": 8, "layer1_order": 2}, {"deep_short_tiles": 0},
                 {"deep_short_tiles": 0, "tile_m": 64}, {"tile_m": 64}):
        print(f"  options {opts}", flush=True)
        run = _run(cfg, inp, ids, w, opts, True)
        np.testing.assert_array_equal(run.out, base.out)


def test_skewed_output_does_not_depend_on_tiling_or_schedule():
    """The skewed workload (one expert with about 26 k rows, Dirichlet segments): every output row of a run with
    128-row tiles in source-segment order equals the default run's, bit for bit."""
    cfg = wl.CONFIGS["skewed"]
    print("skewed variants: generating inputs", flush=True)
    inp = wl.make_inputs(cfg, threads=16)
    ids, w = orc.route_topk(inp.logits, cfg.k)
    base = _run(cfg, inp, ids, w)
    other = _run(cfg, inp, ids, w, {"tile_m": 128, "layer0_order": 1})
    np.testing.assert_array_equal(other.out, base.out)
