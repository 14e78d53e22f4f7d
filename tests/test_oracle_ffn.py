"""Pins of the FFN / combine oracle: hand-computable special cases and library float64
matmuls on the same inputs (the SwiGLU expert FFN and the weighted combine have a plain
definition, so the oracle is that definition; numpy's matmul re-derives it independently)."""
import math

import numpy as np
import pytest

from paper_2512_09277_amd import workloads as W


def silu(v):
    return v / (1.0 + np.exp(-v))


def test_scalar_case(oracle):
    """H = I = 1: y = silu(x*wg) * (x*wu) * wd, computed by hand for x=2, wg=0.5, wu=3, wd=-4."""
    x = np.array([[2.0]], np.float32)
    w13 = np.array([[[0.5], [3.0]]], np.float32)          # [spr=1, 2I=2, H=1]
    w2 = np.array([[[-4.0]]], np.float32)
    y, act = oracle.ffn(x, np.array([0]), np.array([0, 1]), 1, w13, w2, want_act=True)
    gate = 1.0
    expect_act = gate / (1.0 + math.exp(-1.0)) * 6.0       # silu(1) * 6
    assert act[0, 0] == pytest.approx(expect_act, rel=1e-15)
    assert y[0, 0] == pytest.approx(-4.0 * expect_act, rel=1e-15)
    assert expect_act == pytest.approx(4.386351471, rel=1e-9)   # 6 * 0.7310585786 (sigmoid(1))


def test_one_hot_rows_pick_weight_columns(oracle):
    """x = e_h (one-hot): gate_i = w13[l][i][h], up_i = w13[l][I+i][h]; with w2 = identity-like rows
    the output is the activation vector itself."""
    H, I, spr = 4, 4, 2
    rng = np.random.default_rng(0)
    w13 = rng.standard_normal((spr, 2 * I, H)).astype(np.float32)
    w2 = np.zeros((spr, H, I), np.float32)
    for l in range(spr):
        w2[l] = np.eye(H, I) * (l + 1)
    x = np.eye(H, dtype=np.float32)                        # token t = one-hot t
    perm_pair = np.array([2, 0, 3], np.int32)              # k=1: rows are tokens 2 | 0, 3
    go = np.array([0, 1, 3], np.int32)
    y = oracle.ffn(x, perm_pair, go, 1, w13, w2)
    for r, (t, l) in enumerate([(2, 0), (0, 1), (3, 1)]):
        g = w13[l, :I, t].astype(np.float64)
        u = w13[l, I:, t].astype(np.float64)
        assert np.allclose(y[r], (l + 1) * silu(g) * u, rtol=1e-14, atol=0)


def test_constant_up_projection(oracle):
    """W_up == c: up_i = c * sum(x); W_gate rows equal -> every act_i equal; y[c'] = act * rowsum(w2)."""
    H, I = 8, 5
    x = np.arange(1, H + 1, dtype=np.float32).reshape(1, H) / 8
    w13 = np.empty((1, 2 * I, H), np.float32)
    w13[0, :I] = 0.25
    w13[0, I:] = 0.5
    w2 = np.arange(H * I, dtype=np.float32).reshape(1, H, I) / 16
    y, act = oracle.ffn(x, np.array([0]), np.array([0, 1]), 1, w13, w2, want_act=True)
    sx = float(x.sum())                                    # 4.5
    a = silu(np.float64(0.25 * sx)) * 0.5 * sx
    assert np.allclose(act, a, rtol=1e-14)
    assert np.allclose(y[0], a * w2[0].astype(np.float64).sum(axis=1), rtol=1e-14)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_against_float64_matmul(oracle, dtype):
    """Random ragged groups (including an empty slot and a one-row slot, which is a plain GEMV)."""
    T, k, spr, H, I = 9, 2, 4, 48, 24
    x = W.activations(T, H, 11, dtype)
    w13, w2 = W.expert_weights(spr, H, I, 12, dtype)
    perm_pair = np.array([3, 8, 17, 0, 5, 10, 11], np.int32)
    go = np.array([0, 3, 3, 4, 7], np.int32)               # sizes 3, 0, 1, 3
    wide = (lambda a: a.astype(np.float64)) if dtype == "f32" else (lambda a: W.bf16_bits_to_f32(a).astype(np.float64))
    y, act = oracle.ffn(x, perm_pair, go, k, w13, w2, want_act=True)
    X, W13, W2 = wide(x), wide(w13), wide(w2)
    for l in range(spr):
        rows = range(go[l], go[l + 1])
        if not rows:
            continue
        xs = X[perm_pair[list(rows)] // k]
        gu = xs @ W13[l].T
        a = silu(gu[:, :I]) * gu[:, I:]
        assert np.allclose(act[list(rows)], a, rtol=1e-12, atol=1e-15)
        assert np.allclose(y[list(rows)], a @ W2[l].T, rtol=1e-12, atol=1e-15)
    sub = oracle.ffn(x, perm_pair, go, k, w13, w2, rows=[6, 3])          # row subset, any order
    assert np.array_equal(sub, y[[6, 3]])


def test_transposed_operand_would_fail(oracle):
    """Gate and up halves are distinguishable: swapping them changes the result (silu is not symmetric)."""
    x = np.array([[1.0, 2.0]], np.float32)
    w13 = np.array([[[1.0, 0.0], [0.0, 1.0]]], np.float32)  # gate = x0 = 1, up = x1 = 2
    w2 = np.array([[[1.0], [0.0]]], np.float32)             # [1, H=2, I=1]
    y = oracle.ffn(x, np.array([0]), np.array([0, 1]), 1, w13, w2)
    assert y[0, 0] == pytest.approx(2.0 / (1.0 + math.exp(-1.0)), rel=1e-15)   # silu(1)*2, not silu(2)*1
    assert y[0, 1] == 0.0


def test_unpermute_against_einsum(oracle):
    rng = np.random.default_rng(5)
    T, k, H = 6, 3, 10
    pair_row = np.full((T, k), -1, np.int32)
    chosen = rng.permutation(T * k)[:11]
    pair_row.reshape(-1)[np.sort(chosen)] = rng.permutation(11)
    y = rng.standard_normal((11, H))
    w = W.gating_weights(T, k, 9)
    out = oracle.unpermute(y, pair_row, w)
    mask = pair_row >= 0
    gathered = np.where(mask[..., None], y[np.maximum(pair_row, 0)], 0.0)
    assert np.allclose(out, np.einsum("tk,tkh->th", w.astype(np.float64), gathered), rtol=1e-14, atol=1e-16)
    assert (out[~mask.any(axis=1)] == 0).all()


def test_layer_output_is_routing_invariant(oracle):
    """Summing the per-rank partial outputs over all ranks gives sum_j w[t,j] * FFN_{ids[t,j]}(x_t)
    computed densely per logical expert with float64 matmuls -- the same for METRO and for
    token-balanced routing, since replicas share weights and no pair is dropped (eq. (2))."""
    w = W.TINY
    _, s2e, ids = W.routing_inputs(w)
    x = W.activations(w.T, w.H, w.seed(0, 3), "f32")
    w13, w2 = W.expert_weights(w.N, w.H, w.I, w.seed(0, 2), "f32")
    tw = W.gating_weights(w.T, w.k, w.seed(0, 4))
    X = x.astype(np.float64)
    dense = np.zeros((w.T, w.H))
    for t in range(w.T):
        for j in range(w.k):
            e = ids[t, j]
            gu = W13 = w13[e].astype(np.float64) @ X[t]
            a = silu(gu[:w.I]) * gu[w.I:]
            dense[t] += float(tw[t, j]) * (w2[e].astype(np.float64) @ a)
    for route in (oracle.route_metro, oracle.route_token_balanced):
        ps = route(ids, s2e, w.N, w.G, w.spr)["pair_slot"]
        total = np.zeros((w.T, w.H))
        for g in range(w.G):
            pm = oracle.permute(ps, g, w.spr)
            y = oracle.ffn(x, pm["perm_pair"], pm["group_offsets"], w.k,
                           W.rank_share(w13, s2e, g, w.spr), W.rank_share(w2, s2e, g, w.spr))
            total += oracle.unpermute(y, pm["pair_row"], tw)
        assert np.allclose(total, dense, rtol=1e-11, atol=1e-14)


def test_bf16_helpers_round_to_nearest_even():
    f = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0], np.float32)   # 1+2^-8 ties to even (1.0); 1+3*2^-8 -> 1+2^-6
    b = W.f32_to_bf16_bits(f)
    assert b.tolist() == [0x3F80, 0x3F80, 0x3F82, 0xC020, 0x0000]
    assert W.bf16_bits_to_f32(b).tolist() == [1.0, 1.0, 1.015625, -2.5, 0.0]
