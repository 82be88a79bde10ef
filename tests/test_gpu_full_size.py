"""GPU parity at the full workload sizes, in the launch configuration bench.py times: index outputs compared in
full, layer outputs on sampled tokens the oracle computes one by one (tokens are independent along M)."""
import numpy as np
import pytest

import workloads as wl
from oracle import moe_oracle as orc

pytestmark = pytest.mark.gpu


def _sample_tokens(cfg, offsets, perm, tiles, n_random=48):
    """Tokens behind the first/last row of every expert and of a spread of tiles, plus evenly spaced ones."""
    rows = set()
    for e in range(cfg.E):
        if offsets[e + 1] > offsets[e]:
            rows.update((int(offsets[e]), int(offsets[e + 1]) - 1))
    step = max(1, len(tiles["row0"]) // 24)
    for r0, n in list(zip(tiles["row0"], tiles["rows"]))[::step]:
        rows.update((int(r0), int(r0 + n - 1)))
    toks = {int(perm[r]) // cfg.k for r in rows}
    toks.update(np.linspace(0, cfg.T - 1, n_random).astype(int).tolist())
    return np.array(sorted(toks), dtype=np.int64)


@pytest.mark.parametrize("name", ["mixtral", "qwen2", "phi35", "skewed", "qwen2_table2", "mixtral_tp8"])
def test_full_size_sampled_parity(name):
    import gpu_harness as H
    cfg = wl.CONFIGS[name]
    print(f"full-size parity {name}: generating inputs", flush=True)
    inp = wl.make_inputs(cfg, threads=16)
    ids, w = orc.route_topk(inp.logits, cfg.k)
    layer = H.GpuLayer(cfg, inp, ids, w)
    print("  forward", flush=True)
    layer.forward()
    run = layer.results()
    layer.close()
    assert run.status == 0
    counts, offsets, perm, inv = orc.build_permutation(ids, cfg.E)
    np.testing.assert_array_equal(run.counts, counts)
    np.testing.assert_array_equal(run.offsets, offsets)
    np.testing.assert_array_equal(run.perm, perm)
    np.testing.assert_array_equal(run.inv_perm, inv)
    toks = _sample_tokens(cfg, offsets, perm, run.tiles)
    if name in ("mixtral", "skewed"):
        toks = toks[:: 2]            # the widest experts: keep the oracle's share of the run to seconds
    print(f"  oracle on {len(toks)} sampled tokens", flush=True)
    ref = orc.moe_layer_tokens(toks, inp.x, inp.W1, inp.W2, ids, w, cfg.act)
    a, b = H.error_metrics(run.out[toks], ref)
    print(f"  err {a:.3e} {b:.3e}", flush=True)
    assert a <= H.REL_TOL and b <= H.REL_TOL
    # nothing outside the sample is garbage: finite everywhere, and of the sample's magnitude
    assert np.isfinite(run.out).all()
    assert 0.5 < run.out.std() / ref.std() < 2.0


@pytest.mark.parametrize("name", ["mixtral", "qwen2_table2"])
def test_full_size_token_reversal_moves_every_row_bit_for_bit(name):
    """Every output row is the same sum in the same order wherever its token sits: reversing the token order reverses
    the output rows exactly.  This checks every row of the full-size output, not a sample, against a run in which
    each routed row lands in a different tile and a different position of it."""
    import gpu_harness as H
    cfg = wl.CONFIGS[name]
    print(f"token reversal {name}: generating inputs", flush=True)
    inp = wl.make_inputs(cfg, threads=16)
    ids, w = orc.route_topk(inp.logits, cfg.k)
    layer = H.GpuLayer(cfg, inp, ids, w)
    layer.forward(); base = layer.results(); layer.close()
    assert base.status == 0
    rev = wl.MoEInputs(cfg, np.ascontiguousarray(inp.x[::-1]), inp.W1, inp.W2, np.ascontiguousarray(inp.logits[::-1]),
                       inp.seg_offsets)
    print("  reversed forward", flush=True)
    l2 = H.GpuLayer(cfg, rev, np.ascontiguousarray(ids[::-1]), np.ascontiguousarray(w[::-1]))
    l2.forward(); r2 = l2.results(); l2.close()
    assert r2.status == 0
    np.testing.assert_array_equal(r2.out[::-1], base.out)


def test_full_size_whole_output_against_the_oracle():
    """The Mixtral-shaped workload bench.py times, every output element against the oracle (about 6 TFLOP in fp64 on
    the host: seconds on the GPU machine's cores)."""
    import gpu_harness as H
    cfg = wl.CONFIGS["mixtral"]
    print("whole-output parity mixtral: generating inputs", flush=True)
    inp = wl.make_inputs(cfg, threads=16)
    ids, w = orc.route_topk(inp.logits, cfg.k)
    layer = H.GpuLayer(cfg, inp, ids, w)
    layer.forward(); run = layer.results(); layer.close()
    assert run.status == 0
    print("  oracle on all tokens", flush=True)
    ref = orc.moe_layer(inp.x, inp.W1, inp.W2, ids, w, cfg.act)
    a, b = H.error_metrics(run.out, ref)
    print(f"  err {a:.3e} {b:.3e}", flush=True)
    assert a <= H.REL_TOL and b <= H.REL_TOL
