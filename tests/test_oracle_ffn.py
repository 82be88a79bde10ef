"""Pins for the oracle's bf16 handling, activations, expert FFN and top-k combine (CPU only)."""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moe_oracle as orc
from conftest import read_golden


# ---------------------------------------------------------------- bf16
def _bf16_neighbours(v: float):
    """The two bf16 values bracketing v (v > 0, normal range), as exact Fractions, plus their mantissa parity."""
    e = 0
    f = Fraction(v)
    while f >= 2:
        f /= 2
        e += 1
    while f < 1:
        f *= 2
        e -= 1
    lo_m = int(f * 128)            # 1.mmmmmmm -> integer mantissa with 7 fraction bits
    scale = Fraction(2) ** e / 128
    return lo_m * scale, (lo_m + 1) * scale, lo_m % 2 == 0


@pytest.mark.parametrize("v", [1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -40,
                               1.0 + 2.0 ** -8 - 2.0 ** -40, 3.1415926535, 0.1, 1e-3, 255.5, 65280.0 + 128.0])
def test_bf16_rounding_exact_rationals(v):
    lo, hi, lo_even = _bf16_neighbours(v)
    d_lo, d_hi = Fraction(v) - lo, hi - Fraction(v)
    want = lo if d_lo < d_hi or (d_lo == d_hi and lo_even) else hi
    for sign in (1.0, -1.0):
        got = orc.round_f64_to_bf16(np.array([sign * v]))[0]
        assert Fraction(float(got)) == Fraction(sign) * want


def test_bf16_rounding_matches_torch_on_fp32_values():
    v = wl.normal_f32((4096,), 3, 41, 3.0, threads=1)
    want = torch.from_numpy(v).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(orc.round_f64_to_bf16(v.astype(np.float64)), want)
    bits = orc.f64_to_bf16_bits(v.astype(np.float64))
    np.testing.assert_array_equal(orc.bf16_bits_to_f64(bits), want)
    np.testing.assert_array_equal(bits, wl.f32_to_bf16(v))                # the generator's own rounding agrees
    np.testing.assert_array_equal(wl.bf16_to_f32(bits).astype(np.float64), want)


# ---------------------------------------------------------------- activations
def test_activation_constants():
    for name, x, val in read_golden("activation_constants.txt"):
        x, val = float(x), float(val)
        if name == "gelu":
            got = orc.activation(np.array([[x]]), orc.ACT_GELU)[0, 0]
        else:
            got = orc.activation(np.array([[x, 1.0]]), orc.ACT_SWIGLU)[0, 0]   # up = 1 leaves silu(gate)
        assert got == pytest.approx(val, abs=1e-15)


def test_activation_vs_torch():
    g = wl.normal_f32((64, 32), 5, 42, 2.0, threads=1).astype(np.float64)
    tg = torch.from_numpy(g)
    np.testing.assert_allclose(orc.activation(g, orc.ACT_GELU), torch.nn.functional.gelu(tg).numpy(), atol=1e-14)
    want = (torch.nn.functional.silu(tg[:, :16]) * tg[:, 16:]).numpy()          # [gate | up] halves
    np.testing.assert_allclose(orc.activation(g, orc.ACT_SWIGLU), want, atol=1e-14)


# ---------------------------------------------------------------- FFN + combine
def _small_problem(T, H, F, E, k, act, seed):
    cfg = wl.MoEConfig("case", T=T, H=H, F=F, E=E, k=k, act=act, S=4, seed=seed)
    inp = wl.make_inputs(cfg, threads=1)
    ids, w = orc.route_topk(inp.logits, k)
    return cfg, inp, ids, w


def _round_bf16_frexp(v):
    """bf16 rounding written another way: 8 significant bits via frexp/rint (rint rounds ties to even)."""
    m, e = np.frexp(v)
    return np.ldexp(np.rint(m * 256.0) / 256.0, e)


def _dense_per_token(inp, ids, w, act, round_h):
    """Brute force: no permutation, no grouping.  One token-expert pair at a time."""
    cfg = inp.cfg
    x = wl.bf16_to_f32(inp.x).astype(np.float64)
    W1 = wl.bf16_to_f32(inp.W1).astype(np.float64)
    W2 = wl.bf16_to_f32(inp.W2).astype(np.float64)
    out = np.zeros((cfg.T, cfg.H))
    for t in range(cfg.T):
        for j in range(cfg.k):
            e = int(ids[t, j])
            g = np.array([np.dot(x[t], W1[e][:, c]) for c in range(W1.shape[2])])
            if act == orc.ACT_GELU:
                h = np.array([v * 0.5 * math.erfc(-v / math.sqrt(2.0)) for v in g])   # v * Phi(v)
            elif act == orc.ACT_SWIGLU:
                F = cfg.F
                h = torch.nn.functional.silu(torch.from_numpy(g[:F])).numpy() * g[F:]
            else:
                h = g
            if round_h:
                h = _round_bf16_frexp(h)
            y = np.array([np.dot(h, W2[e][:, c]) for c in range(cfg.H)])
            out[t] += float(w[t, j]) * y
    return out


@pytest.mark.parametrize("act", [orc.ACT_GELU, orc.ACT_SWIGLU, orc.ACT_IDENTITY])
def test_layer_vs_per_token_bruteforce(act):
    cfg, inp, ids, w = _small_problem(T=24, H=16, F=24, E=4, k=2, act=act, seed=21)
    got = orc.moe_layer(inp.x, inp.W1, inp.W2, ids, w, act, round_h=False)
    want = _dense_per_token(inp, ids, w, act, round_h=False)
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-12)
    # with the bf16 rounding of h: a different summation order can flip a borderline rounding of single
    # h elements, each worth at most |h| 2^-8 |W2|; everything else must agree to fp64 accuracy.
    got_r = orc.moe_layer(inp.x, inp.W1, inp.W2, ids, w, act, round_h=True)
    want_r = _dense_per_token(inp, ids, w, act, round_h=True)
    diff = np.abs(got_r - want_r)
    assert (diff > 1e-10).mean() < 0.02 and diff.max() < 2e-3
    assert np.abs(got_r - got).max() > 1e-6          # the rounding is really applied ...
    assert np.abs(got_r - got).max() < 5e-2          # ... and is a small perturbation


@pytest.mark.parametrize("act", [orc.ACT_GELU, orc.ACT_SWIGLU])
def test_single_expert_is_a_dense_mlp(act):
    cfg, inp, _, _ = _small_problem(T=40, H=48, F=80, E=1, k=1, act=act, seed=22)
    ids = np.zeros((cfg.T, 1), np.int32)
    w = np.ones((cfg.T, 1), np.float32)
    got = orc.moe_layer(inp.x, inp.W1, inp.W2, ids, w, act, round_h=False)
    x = torch.from_numpy(wl.bf16_to_f32(inp.x)).double()
    W1 = torch.from_numpy(wl.bf16_to_f32(inp.W1[0])).double()
    W2 = torch.from_numpy(wl.bf16_to_f32(inp.W2[0])).double()
    G = x @ W1
    h = torch.nn.functional.gelu(G) if act == orc.ACT_GELU else torch.nn.functional.silu(G[:, :cfg.F]) * G[:, cfg.F:]
    np.testing.assert_allclose(got, (h @ W2).numpy(), rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("act", [orc.ACT_GELU, orc.ACT_SWIGLU])
def test_column_chunks_narrower_than_the_layer(act):
    """The expert FFN walks W1's columns and W2's rows in chunks; with chunks narrower than F (and a ragged last
    one) the result is still the dense two-layer MLP of a library matmul."""
    cfg, inp, _, _ = _small_problem(T=20, H=32, F=88, E=2, k=1, act=act, seed=27)
    ids = (np.arange(cfg.T) % 2).astype(np.int32).reshape(-1, 1)
    _, offsets, perm, _ = orc.build_permutation(ids, cfg.E)
    x = torch.from_numpy(wl.bf16_to_f32(inp.x)).double()
    for chunk in (24, 40, 4096):
        Y = orc.expert_ffn(inp.x, inp.W1, inp.W2, offsets, perm, 1, act, round_h=False, col_chunk=chunk)
        for e in range(cfg.E):
            W1 = torch.from_numpy(wl.bf16_to_f32(inp.W1[e])).double()
            W2 = torch.from_numpy(wl.bf16_to_f32(inp.W2[e])).double()
            G = x[e::2] @ W1
            h = torch.nn.functional.gelu(G) if act == orc.ACT_GELU else torch.nn.functional.silu(G[:, :cfg.F]) * G[:, cfg.F:]
            np.testing.assert_allclose(Y[offsets[e]:offsets[e + 1]], (h @ W2).numpy(), rtol=1e-11, atol=1e-12)


def test_identity_activation_makes_the_layer_linear():
    cfg, inp, ids, w = _small_problem(T=30, H=20, F=36, E=5, k=3, act=orc.ACT_IDENTITY, seed=23)
    got = orc.moe_layer(inp.x, inp.W1, inp.W2, ids, w, orc.ACT_IDENTITY, round_h=False)
    x = wl.bf16_to_f32(inp.x).astype(np.float64)
    P = [wl.bf16_to_f32(inp.W1[e]).astype(np.float64) @ wl.bf16_to_f32(inp.W2[e]).astype(np.float64)
         for e in range(cfg.E)]                                            # (x W1) W2 = x (W1 W2)
    want = np.stack([sum(float(w[t, j]) * (x[t] @ P[int(ids[t, j])]) for j in range(cfg.k)) for t in range(cfg.T)])
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-11)


def test_all_experts_equal_weights_is_the_mean():
    cfg, inp, _, _ = _small_problem(T=12, H=16, F=20, E=4, k=4, act=orc.ACT_GELU, seed=24)
    ids = np.tile(np.array([2, 0, 3, 1], np.int32), (cfg.T, 1))
    w = np.full((cfg.T, 4), 0.25, np.float32)
    got = orc.moe_layer(inp.x, inp.W1, inp.W2, ids, w, orc.ACT_GELU, round_h=False)
    x = torch.from_numpy(wl.bf16_to_f32(inp.x)).double()
    outs = []
    for e in range(4):
        W1 = torch.from_numpy(wl.bf16_to_f32(inp.W1[e])).double()
        W2 = torch.from_numpy(wl.bf16_to_f32(inp.W2[e])).double()
        outs.append(torch.nn.functional.gelu(x @ W1) @ W2)
    np.testing.assert_allclose(got, torch.stack(outs).mean(0).numpy(), rtol=1e-11, atol=1e-12)


def test_token_permutation_and_subsets():
    cfg, inp, ids, w = _small_problem(T=50, H=32, F=40, E=6, k=2, act=orc.ACT_SWIGLU, seed=25)
    full = orc.moe_layer(inp.x, inp.W1, inp.W2, ids, w, cfg.act)
    p = np.random.default_rng(0).permutation(cfg.T)
    shuffled = orc.moe_layer(inp.x[p], inp.W1, inp.W2, ids[p], w[p], cfg.act)
    np.testing.assert_allclose(shuffled, full[p], rtol=1e-12, atol=1e-13)
    sub = [3, 49, 0, 17]
    np.testing.assert_allclose(orc.moe_layer_tokens(sub, inp.x, inp.W1, inp.W2, ids, w, cfg.act), full[sub],
                               rtol=1e-12, atol=1e-13)


def test_combine_uses_the_right_slot_weights():
    # Y rows are one-hot in the pair id, so out[t] lists w[t,j] at column t*k+j and nothing else.
    T, k, E = 6, 3, 4
    ids = np.array([[(t + j) % E for j in range(k)] for t in range(T)], np.int32)
    w = (np.arange(T * k, dtype=np.float32).reshape(T, k) + 1) / 100
    _, _, perm, inv = orc.build_permutation(ids, E)
    Y = np.zeros((T * k, T * k))
    Y[np.arange(T * k), perm] = 1.0
    out = orc.combine(Y, inv, w)
    want = np.zeros((T, T * k))
    for t in range(T):
        for j in range(k):
            want[t, t * k + j] = w[t, j]
    np.testing.assert_array_equal(out, want.astype(np.float64))


def test_tiny_config_sanity():
    cfg = wl.CONFIGS["tiny"]
    inp = wl.make_inputs(cfg, threads=1)
    ids, w = orc.route_topk(inp.logits, cfg.k)
    out = orc.moe_layer(inp.x, inp.W1, inp.W2, ids, w, cfg.act)
    assert out.shape == (cfg.T, cfg.H) and np.isfinite(out).all()
    # unit-variance inputs and 1/sqrt(fan_in) weights keep the output O(1)
    assert 0.05 < out.std() < 2.0
