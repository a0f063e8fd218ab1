"""Pins for oracle.attention, oracle.pointwise and oracle.layers (textbook definitions)."""
import math
import os

import numpy as np
import pytest

import hapgen
from oracle import attention, pointwise, layers

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _qkv(b=2, h=3, s=7, d=4, seed=2):
    mk = lambda t: hapgen.normal(seed, t, (b, h, s, d))
    return mk(hapgen.TensorId.Q), mk(hapgen.TensorId.K), mk(hapgen.TensorId.V), mk(hapgen.TensorId.DO)


def test_attention_brute_force_loops():
    Q, K, V, _ = _qkv(b=1, h=2, s=5, d=3)
    O, lse = attention.attn_fwd(Q, K, V)
    for h in range(2):
        for q in range(5):
            sc = [sum(Q[0, h, q, x] * K[0, h, k, x] for x in range(3)) / math.sqrt(3) for k in range(5)]
            den = sum(math.exp(v) for v in sc)
            assert lse[0, h, q] == pytest.approx(math.log(den), abs=1e-12)
            for x in range(3):
                assert O[0, h, q, x] == pytest.approx(sum(math.exp(sc[k]) / den * V[0, h, k, x] for k in range(5)), abs=1e-12)


def test_attention_special_cases():
    Q, K, V, _ = _qkv()
    O, _ = attention.attn_fwd(Q, K, np.ones_like(V))          # rows of P sum to one
    assert np.allclose(O, 1.0, atol=1e-14)
    O, _ = attention.attn_fwd(np.zeros_like(Q), K, V)         # uniform P -> mean over keys
    assert np.allclose(O, np.broadcast_to(V.mean(axis=2, keepdims=True), V.shape), atol=1e-14)
    perm = np.random.default_rng(0).permutation(K.shape[2])   # keys and values permuted together
    O1, _ = attention.attn_fwd(Q, K, V); O2, _ = attention.attn_fwd(Q, K[:, :, perm], V[:, :, perm])
    assert np.allclose(O1, O2, atol=1e-13)
    # head / batch slices are independent
    offs = [0, 1, 3]
    parts = [attention.attn_fwd(*(attention.slice_heads_or_batch(t, True, offs, j) for t in (Q, K, V)))[0] for j in range(2)]
    assert np.allclose(np.concatenate(parts, 1), O1, atol=1e-14)
    offs = [0, 2, 2]
    parts = [attention.attn_fwd(*(attention.slice_heads_or_batch(t, False, offs, j) for t in (Q, K, V)))[0] for j in range(2)]
    assert np.allclose(np.concatenate(parts, 0), O1, atol=1e-14)


def test_attention_backward_finite_differences():
    Q, K, V, dO = _qkv(b=1, h=2, s=6, d=4)
    dQ, dK, dV = attention.attn_bwd(Q, K, V, dO)
    L = lambda q, k, v: float((attention.attn_fwd(q, k, v)[0] * dO).sum())
    h = 1e-6
    for idx in [(0, 0, 0, 0), (0, 1, 3, 2), (0, 1, 5, 3)]:
        for which, g in enumerate((dQ, dK, dV)):
            args_p = [Q.copy(), K.copy(), V.copy()]; args_m = [Q.copy(), K.copy(), V.copy()]
            args_p[which][idx] += h; args_m[which][idx] -= h
            assert (L(*args_p) - L(*args_m)) / (2 * h) == pytest.approx(g[idx], rel=1e-6, abs=1e-8)


def test_gelu_table_limits_and_derivative():
    with open(os.path.join(GOLD, "gelu_table.txt")) as f:
        for l in f:
            if l.strip() and not l.startswith("#"):
                x, y = map(float, l.split())
                assert float(pointwise.gelu(np.float64(x))) == pytest.approx(y, abs=2e-10)
    assert float(pointwise.gelu(np.float64(30.0))) == 30.0
    assert abs(float(pointwise.gelu(np.float64(-30.0)))) < 1e-100
    x = np.linspace(-4, 4, 41); h = 1e-6
    assert np.allclose((pointwise.gelu(x + h) - pointwise.gelu(x - h)) / (2 * h), pointwise.gelu_grad(x), atol=1e-8)


def test_layernorm_properties_and_finite_differences():
    x = hapgen.normal(4, hapgen.TensorId.X, (5, 16)) * 3 + 1
    g = hapgen.normal(4, hapgen.TensorId.GAMMA, (16,)) + 1; b = hapgen.normal(4, hapgen.TensorId.BETA, (16,))
    y, mu, rstd = pointwise.layernorm_fwd(x, 1.0, 0.0)
    assert np.allclose(y.mean(-1), 0, atol=1e-13)
    assert np.allclose((y ** 2).mean(-1), x.var(-1) / (x.var(-1) + 1e-5), atol=1e-12)
    dy = hapgen.normal(4, hapgen.TensorId.DY, (5, 16))
    dx, dg, db = pointwise.layernorm_bwd(x, g, dy)
    L = lambda x_, g_, b_: float((pointwise.layernorm_fwd(x_, g_, b_)[0] * dy).sum())
    h = 1e-6
    for (r, c) in [(0, 0), (2, 7), (4, 15)]:
        xp, xm = x.copy(), x.copy(); xp[r, c] += h; xm[r, c] -= h
        assert (L(xp, g, b) - L(xm, g, b)) / (2 * h) == pytest.approx(dx[r, c], rel=1e-5, abs=1e-8)
    for c in [0, 9]:
        gp, gm = g.copy(), g.copy(); gp[c] += h; gm[c] -= h
        assert (L(x, gp, b) - L(x, gm, b)) / (2 * h) == pytest.approx(dg[c], rel=1e-6, abs=1e-8)
    assert np.allclose(db, dy.sum(0))


def _enc_params(H, F, seed=6):
    T = hapgen.TensorId
    p = dict(Wq=hapgen.normal(seed, T.WQ, (H, H), .3), Wk=hapgen.normal(seed, T.WK, (H, H), .3),
             Wv=hapgen.normal(seed, T.WV, (H, H), .3), Wo=hapgen.normal(seed, T.WO, (H, H), .3),
             W1=hapgen.normal(seed, T.W, (H, F), .3), W2=hapgen.normal(seed, T.W2, (F, H), .3))
    for i, (n, sz) in enumerate([("bq", H), ("bk", H), ("bv", H), ("bo", H), ("b1", F), ("b2", H), ("be1", H), ("be2", H)]):
        p[n] = hapgen.normal(seed, T.MISC + i, (sz,), .2)
    p["g1"] = 1 + hapgen.normal(seed, T.MISC + 20, (H,), .2); p["g2"] = 1 + hapgen.normal(seed, T.MISC + 21, (H,), .2)
    return p


def test_encoder_layer_and_mlp_finite_differences():
    B, S, heads, d, F = 2, 3, 2, 4, 10
    H = heads * d
    p = _enc_params(H, F)
    x = hapgen.normal(6, hapgen.TensorId.X, (B * S, H)); dY = hapgen.normal(6, hapgen.TensorId.DY, (B * S, H))
    r = layers.encoder_layer(x, p, dY, B, S, heads, d)
    L = lambda x_, p_: float((layers.encoder_layer(x_, p_, dY, B, S, heads, d)["y"] * dY).sum())
    h = 1e-6
    for idx in [(0, 0), (3, 5), (5, 7)]:
        xp, xm = x.copy(), x.copy(); xp[idx] += h; xm[idx] -= h
        assert (L(xp, p) - L(xm, p)) / (2 * h) == pytest.approx(r["dx"][idx], rel=2e-5, abs=1e-7)
    for name in ["Wq", "Wk", "Wv", "Wo", "W1", "W2", "bq", "bk", "bv", "bo", "b1", "b2", "g1", "be1", "g2", "be2"]:
        idx = tuple(s // 2 for s in p[name].shape)
        pp = {k: v.copy() for k, v in p.items()}; pm = {k: v.copy() for k, v in p.items()}
        pp[name][idx] += h; pm[name][idx] -= h
        assert (L(x, pp) - L(x, pm)) / (2 * h) == pytest.approx(r["d" + name][idx], rel=2e-5, abs=1e-7), name
    m = layers.mlp_block(x, p["W1"], p["b1"], p["W2"], p["b2"], dY)
    Lm = lambda x_: float((layers.mlp_block(x_, p["W1"], p["b1"], p["W2"], p["b2"], dY)["out"] * dY).sum())
    xp, xm = x.copy(), x.copy(); xp[1, 2] += h; xm[1, 2] -= h
    assert (Lm(xp) - Lm(xm)) / (2 * h) == pytest.approx(m["dX"][1, 2], rel=1e-5, abs=1e-8)
