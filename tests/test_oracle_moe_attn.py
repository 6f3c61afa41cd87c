"""Pins for the oracle's MoE FFN, bf16 rounding and sparse attention (no GPU)."""
import math

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

from oracle import pit_oracle as orc
from paper_2301_10936_amd import workloads as wl


# ---------------------------------------------------------------- bf16 rounding
def test_round_to_bf16_known_values():
    x = np.array([1.0, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -20, -1 - 2.0 ** -8,
                  0.0, 3.0, 2.0 ** -126 * 1.5, 2.0 ** -133, 2.0 ** -134, 1.7014118e38])
    want = np.array([1.0, 1.0, 1 + 2.0 ** -6, 1 + 2.0 ** -7, -1.0,
                     0.0, 3.0, 2.0 ** -126 * 1.5, 2.0 ** -133, 0.0, 1.7014118346046923e38])
    assert np.array_equal(orc.round_to_bf16(x), want)


def test_round_to_bf16_agrees_with_independent_bit_trick():
    g = np.random.default_rng(0)
    x = (g.standard_normal(200000) * np.exp(g.uniform(-20, 20, 200000))).astype(np.float32)
    via_bits = orc.bf16_bits_to_f64(wl.to_bf16_bits(x))           # generator's add-0x7FFF trick
    assert np.array_equal(orc.round_to_bf16(x.astype(np.float64)), via_bits)
    assert np.array_equal(orc.round_to_bf16(via_bits), via_bits)  # idempotent


# ---------------------------------------------------------------- GELU
def test_gelu_closed_forms():
    assert orc.gelu(np.array([0.0]))[0] == 0.0
    assert math.isclose(orc.gelu(np.array([1.0]))[0], 0.8413447460685429, rel_tol=1e-15)
    assert math.isclose(orc.gelu(np.array([-1.0]))[0], -0.15865525393145707, rel_tol=1e-14)
    x = np.linspace(-6, 6, 101)
    assert np.allclose(orc.gelu(x) - orc.gelu(-x), x, atol=1e-15)         # x*Phi(x) + x*Phi(-x) = x
    assert np.allclose(orc.gelu(np.array([30.0, -30.0])), [30.0, 0.0], atol=1e-15)


# ---------------------------------------------------------------- MoE
def test_single_expert_is_a_plain_ffn():
    w = wl.moe_ffn(T=24, d_model=16, d_ff=40, E=1, seed=1, unit_gate=True)
    Y = orc.moe_ffn(w.X, w.expert_id, None, w.W1, w.W2, round_hidden=False)
    X, W1, W2 = orc.to_f64(w.X), orc.to_f64(w.W1[0]), orc.to_f64(w.W2[0])
    H = X @ W1
    ref = (H * 0.5 * (1 + np.vectorize(math.erf)(H / math.sqrt(2)))) @ W2
    assert np.allclose(Y, ref, rtol=1e-13, atol=1e-15)


def test_moe_bruteforce_loops():
    w = wl.moe_ffn(T=6, d_model=4, d_ff=5, E=3, seed=2, w_std=0.5)
    Y = orc.moe_ffn(w.X, w.expert_id, w.gate, w.W1, w.W2, round_hidden=False)
    X, W1, W2 = orc.to_f64(w.X), orc.to_f64(w.W1), orc.to_f64(w.W2)
    for t in range(6):
        e = int(w.expert_id[t])
        h = [sum(X[t, k] * W1[e, k, f] for k in range(4)) for f in range(5)]
        h = [0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in h]
        for n in range(4):
            y = float(w.gate[t]) * sum(h[f] * W2[e, f, n] for f in range(5))
            assert math.isclose(Y[t, n], y, rel_tol=1e-12, abs_tol=1e-15)


def test_moe_routing_properties():
    w = wl.moe_ffn(T=40, d_model=8, d_ff=16, E=4, seed=3, w_std=0.3)
    Y = orc.moe_ffn(w.X, w.expert_id, w.gate, w.W1, w.W2)
    # token permutation permutes the output rows (tokens are a PIT-axis)
    p = np.random.default_rng(0).permutation(40)
    Yp = orc.moe_ffn(w.X[p], w.expert_id[p], w.gate[p], w.W1, w.W2)
    assert np.array_equal(Yp, Y[p])
    # a token only sees its own expert: wreck expert 2's weights, other tokens unchanged
    W1b = w.W1.copy()
    W1b[2] = 0x7FC0
    Yb = orc.moe_ffn(w.X, w.expert_id, w.gate, W1b, w.W2)
    other = w.expert_id != 2
    assert np.array_equal(Yb[other], Y[other]) and np.isnan(Yb[~other]).all()
    # gate scales linearly
    Y1 = orc.moe_ffn(w.X, w.expert_id, None, w.W1, w.W2)
    assert np.allclose(Y, Y1 * w.gate[:, None], rtol=1e-15)
    # hidden rounding: rounded and unrounded differ, but by no more than bf16 spacing allows
    Yu = orc.moe_ffn(w.X, w.expert_id, w.gate, w.W1, w.W2, round_hidden=False)
    assert not np.array_equal(Yu, Y)
    assert orc.rel_errors(Y, Yu)[1] < 2.0 ** -8


def test_moe_identity_activation_on_integers_is_exact():
    w = wl.moe_ffn(T=16, d_model=8, d_ff=8, E=2, seed=4, integer=True, unit_gate=True)
    Y = orc.moe_ffn(w.X, w.expert_id, None, w.W1, w.W2, activation="identity")
    X, W1, W2 = orc.to_f64(w.X), orc.to_f64(w.W1), orc.to_f64(w.W2)
    for t in range(16):
        e = w.expert_id[t]
        assert np.array_equal(Y[t], (X[t] @ W1[e]) @ W2[e])
    assert np.array_equal(Y, np.rint(Y))


def test_zipf_routing_recipe():
    w = wl.moe_ffn(T=4096, d_model=8, d_ff=8, E=64, seed=None)
    cnt = np.bincount(w.expert_id, minlength=64)
    assert cnt.sum() == 4096 and cnt.max() > 700 and cnt.min() < 40


# ---------------------------------------------------------------- attention
def test_full_mask_is_standard_attention():
    w = wl.sparse_attn(H=2, S=24, D=8, window=4, qblock=8, density=0.1, seed=1)
    full = np.ones((24, 24), dtype=np.uint8)
    O = orc.sparse_attn(w.Q, w.K, w.V, full, w.scale)
    Q, K, V = orc.to_f64(w.Q), orc.to_f64(w.K), orc.to_f64(w.V)
    for h in range(2):
        ref = sp_softmax(Q[h] @ K[h].T * w.scale, axis=1) @ V[h]
        assert np.allclose(O[h], ref, rtol=1e-12, atol=1e-14)


def test_attention_bruteforce_loops():
    w = wl.sparse_attn(H=1, S=8, D=4, window=2, qblock=4, density=0.3, seed=2)
    O = orc.sparse_attn(w.Q, w.K, w.V, w.mask, w.scale)
    Q, K, V = orc.to_f64(w.Q)[0], orc.to_f64(w.K)[0], orc.to_f64(w.V)[0]
    for i in range(8):
        ws = {}
        for j in range(8):
            if w.mask[i, j]:
                ws[j] = math.exp(w.scale * sum(Q[i, d] * K[j, d] for d in range(4)))
        z = sum(ws.values())
        for d in range(4):
            ref = sum(ws[j] * V[j, d] for j in ws) / z
            assert math.isclose(O[0, i, d], ref, rel_tol=1e-12, abs_tol=1e-14)


def test_attention_special_cases():
    w = wl.sparse_attn(H=1, S=16, D=8, window=4, qblock=8, density=0.2, seed=3)
    V = orc.to_f64(w.V)
    # one allowed key per query -> that key's value row, exactly
    m = np.zeros((16, 16), dtype=np.uint8)
    tgt = (np.arange(16) * 5) % 16
    m[np.arange(16), tgt] = 1
    assert np.array_equal(orc.sparse_attn(w.Q, w.K, w.V, m, w.scale)[0], V[0][tgt])
    # Q = 0 -> uniform average over the allowed keys
    Oz = orc.sparse_attn(np.zeros_like(w.Q), w.K, w.V, w.mask, w.scale)[0]
    for i in range(16):
        assert np.allclose(Oz[i], V[0][w.mask[i] != 0].mean(0), rtol=1e-13)
    # V = 1 -> rows of ones (softmax weights sum to one); an empty row gives zeros
    m2 = w.mask.copy()
    m2[5] = 0
    ones = np.full_like(w.V, 0x3F80)
    O1 = orc.sparse_attn(w.Q, w.K, ones, m2, w.scale)[0]
    assert np.allclose(np.delete(O1, 5, 0), 1.0, rtol=1e-14) and np.all(O1[5] == 0)
    # keys outside the mask cannot influence the result
    K2 = w.K.copy()
    dead = ~(w.mask != 0).any(axis=0)
    K2[0, dead] = 0x7FC0
    assert np.array_equal(orc.sparse_attn(w.Q, K2, w.V, w.mask, w.scale), orc.sparse_attn(w.Q, w.K, w.V, w.mask, w.scale))
    # scale matters (a dropped scale must be caught)
    assert not np.allclose(orc.sparse_attn(w.Q, w.K, w.V, w.mask, 1.0), orc.sparse_attn(w.Q, w.K, w.V, w.mask, w.scale))


def test_attention_mask_recipe():
    w = wl.sparse_attn(H=1, S=4096, D=8, seed=None)
    sp, ix, bits = orc.build_index(w.mask, 32, 1, 1)
    per_block = np.diff(sp)
    assert 400 < per_block.mean() < 520            # band (~287 key columns) + 5% of the rest
    assert np.all(np.diag(w.mask) == 1)
    i, j = 1000, 1128
    assert w.mask[i, j] == 1 and (w.mask[i, j + 1] == 1) == bool(w.mask[i - i % 32:i - i % 32 + 32, j + 1].all())
