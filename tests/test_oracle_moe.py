"""Pins for oracle.moe (Sec. 7.6: experts of an MoE layer placed unevenly over the devices)."""
import numpy as np
import pytest

import hapgen
from hapgen import TensorId as T
from oracle import linear, lp, moe, rounding


def _data(E=5, C=7, I=6, O=4, seed=11):
    X = hapgen.normal(seed, T.X, (E, C, I))
    W = hapgen.normal(seed, T.W, (E, I, O), 0.4)
    b = hapgen.normal(seed, T.BIAS, (E, O), 0.5)
    dY = hapgen.normal(seed, T.DY, (E, C, O))
    return X, W, b, dY


def test_brute_force_loops_exact_on_integers():
    rng = np.random.default_rng(1)
    E, C, I, O = 3, 4, 5, 2
    X = rng.integers(-3, 4, (E, C, I)).astype(float); W = rng.integers(-3, 4, (E, I, O)).astype(float)
    b = rng.integers(-3, 4, (E, O)).astype(float); dY = rng.integers(-3, 4, (E, C, O)).astype(float)
    rows = [4, 0, 3]
    Y, pre = moe.moe_linear_fwd(X, W, b, rows)
    dX, dW, db = moe.moe_linear_bwd(X, W, pre, dY, rows)
    for e in range(E):
        for t in range(C):
            live = t < rows[e]
            for o in range(O):
                assert Y[e, t, o] == ((sum(X[e, t, i] * W[e, i, o] for i in range(I)) + b[e, o]) if live else 0)
            for i in range(I):
                assert dX[e, t, i] == (sum(dY[e, t, o] * W[e, i, o] for o in range(O)) if live else 0)
        for i in range(I):
            for o in range(O):
                assert dW[e, i, o] == sum(X[e, t, i] * dY[e, t, o] for t in range(rows[e]))
        for o in range(O):
            assert db[e, o] == sum(dY[e, t, o] for t in range(rows[e]))


@pytest.mark.parametrize("act", [False, True])
def test_dispatch_expert_combine_equals_dense_gated_sum(act):
    """Top-1 routing: y_t = sum_e G[t,e] * f_e(x_t) with a one-hot gate G, evaluated densely (every token through
    every expert) and through the dispatched buffers, must agree: pins the expert index of every operand."""
    E, C, I, O, Tn = 4, 6, 5, 3, 15
    _, W, b, _ = _data(E, C, I, O)
    x = hapgen.normal(5, T.X, (Tn, I))
    choice = np.array([0, 2, 2, 1, 3, 0, 2, 1, 1, 0, 3, 2, 0, 2, 2])          # expert of every token (2 gets 6 = C tokens)
    dense = np.stack([linear.linear_fwd(x, W[e], b[e], act)[0] for e in range(E)], axis=1)   # [T, E, O]
    want = dense[np.arange(Tn), choice]
    # dispatch: token t goes to the next free row of its expert's buffer; unused rows are poisoned
    X = np.full((E, C, I), np.nan); rows = np.zeros(E, dtype=int); slot = np.zeros(Tn, dtype=int)
    for t in range(Tn):
        e = choice[t]; slot[t] = rows[e]; X[e, rows[e]] = x[t]; rows[e] += 1
    Y, _ = moe.moe_linear_fwd(X, W, b, rows, act)
    assert np.isfinite(Y).all()                                                # rows without a token are never read
    got = Y[choice, slot]
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-13)


def test_shared_weights_reduce_to_one_linear_layer():
    """If every expert holds the same W and b, the layer is one fully-connected layer over all dispatched tokens."""
    X, W, b, dY = _data()
    E, C, I = X.shape
    rows = [7, 3, 0, 5, 1]
    Ws = np.broadcast_to(W[0], W.shape); bs = np.broadcast_to(b[0], b.shape)
    Y, pre = moe.moe_linear_fwd(X, Ws, bs, rows, act=True)
    dX, dW, db = moe.moe_linear_bwd(X, Ws, pre, dY, rows, act=True)
    live = np.concatenate([np.arange(C) < r for r in rows])
    Xf, dYf = X.reshape(E * C, I)[live], dY.reshape(E * C, -1)[live]
    Yl, prel = linear.linear_fwd(Xf, W[0], b[0], act=True)
    dXl, dWl, dbl = linear.linear_bwd(Xf, W[0], prel, dYf, act=True)
    np.testing.assert_allclose(Y.reshape(E * C, -1)[live], Yl, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(dX.reshape(E * C, -1)[live], dXl, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(dW.sum(axis=0), dWl, rtol=1e-12, atol=1e-12)   # the experts' dW are partials of the one layer's
    np.testing.assert_allclose(db.sum(axis=0), dbl, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("act", [False, True])
def test_finite_differences(act):
    X, W, b, dY = _data()
    rows = [7, 2, 0, 6, 4]
    _, pre = moe.moe_linear_fwd(X, W, b, rows, act)
    dX, dW, db = moe.moe_linear_bwd(X, W, pre, dY, rows, act)
    L = lambda X_, W_, b_: float((moe.moe_linear_fwd(X_, W_, b_, rows, act)[0] * dY).sum())
    h = 1e-6
    for idx in [(0, 0, 0), (1, 1, 5), (3, 5, 2), (4, 3, 4), (1, 2, 0), (2, 0, 0)]:    # the last two are rows without a token
        Xp, Xm = X.copy(), X.copy(); Xp[idx] += h; Xm[idx] -= h
        assert (L(Xp, W, b) - L(Xm, W, b)) / (2 * h) == pytest.approx(dX[idx], rel=1e-6, abs=1e-7)
    for idx in [(0, 0, 0), (1, 5, 3), (2, 1, 1), (4, 2, 2)]:                          # expert 2 has no token: dW = 0
        Wp, Wm = W.copy(), W.copy(); Wp[idx] += h; Wm[idx] -= h
        assert (L(X, Wp, b) - L(X, Wm, b)) / (2 * h) == pytest.approx(dW[idx], rel=1e-6, abs=1e-7)
    for idx in [(0, 0), (3, 3), (2, 1)]:
        bp, bm = b.copy(), b.copy(); bp[idx] += h; bm[idx] -= h
        assert (L(X, W, bp) - L(X, W, bm)) / (2 * h) == pytest.approx(db[idx], rel=1e-6, abs=1e-7)
    assert not dW[2].any() and not db[2].any() and not dX[1, 2:].any()


def test_uneven_expert_placement_tiles_the_layer():
    """Any integer split of the expert axis - here the LP + rounding result for unequal devices, with a device that
    owns no expert - reproduces the unsharded layer by concatenation, with no padded expert."""
    X, W, b, dY = _data(E=7)
    rows = [7, 5, 0, 7, 1, 6, 3]
    speeds = (1.0, 1.0, 0.5, 0.5, 0.01)
    ratios, _ = lp.shard_ratios(speeds, [(1.0, 0, 0, 0)])
    sizes, offs = rounding.round_shards(ratios, 7, 1)
    assert sizes == [3, 2, 1, 1, 0] and offs == [0, 3, 5, 6, 7, 7]
    Y, pre = moe.moe_linear_fwd(X, W, b, rows, act=True)
    dX, dW, db = moe.moe_linear_bwd(X, W, pre, dY, rows, act=True)
    Ys, dXs, dWs, dbs = [], [], [], []
    for j in range(len(speeds)):
        yj, pj = moe.sharded_moe_linear_fwd(offs, j, X, W, b, rows, act=True)
        assert yj.shape[0] == sizes[j]
        a, c, d = moe.sharded_moe_linear_bwd(offs, j, X, W, pre, dY, rows, act=True)
        Ys.append(yj); dXs.append(a); dWs.append(c); dbs.append(d)
    assert np.array_equal(np.concatenate(Ys), Y) and np.array_equal(np.concatenate(dXs), dX)
    assert np.array_equal(np.concatenate(dWs), dW) and np.array_equal(np.concatenate(dbs), db)


def test_padded_expert_changes_nothing_and_full_capacity_default():
    """The padding an even split needs (experts that receive no token) contributes zeros: what the uneven split saves is
    pure overhead.  rows=None means every buffer row holds a token."""
    X, W, b, dY = _data(E=3)
    Xp = np.concatenate([X, np.full((1,) + X.shape[1:], np.nan)]); Wp = np.concatenate([W, W[:1]])
    bp = np.concatenate([b, b[:1]]); dYp = np.concatenate([dY, np.full((1,) + dY.shape[1:], np.nan)])
    rows = [7, 7, 7]
    Y, pre = moe.moe_linear_fwd(X, W, b)
    Yp, prep = moe.moe_linear_fwd(Xp, Wp, bp, rows + [0])
    assert np.array_equal(Yp[:3], Y) and not Yp[3].any()
    dX, dW, db = moe.moe_linear_bwd(X, W, pre, dY)
    dXp, dWp, dbp = moe.moe_linear_bwd(Xp, Wp, prep, dYp, rows + [0])
    assert np.array_equal(dXp[:3], dX) and np.array_equal(dWp[:3], dW) and not dWp[3].any() and not dbp[3].any()
    with pytest.raises(ValueError):
        moe.moe_linear_fwd(X, W, b, [8, 0, 0])


def test_expert_ffn_block_is_one_mlp_block_per_expert():
    """The two-layer expert block composes the per-expert layers: each expert equals the (separately pinned) dense MLP
    block on its own tokens, and the block's dX matches finite differences through both layers."""
    from oracle import layers
    E, C, Hd, F = 4, 6, 5, 7
    X = hapgen.normal(2, T.X, (E, C, Hd)); dOut = hapgen.normal(2, T.DY, (E, C, Hd))
    W1 = hapgen.normal(2, T.W, (E, Hd, F), 0.4); b1 = hapgen.normal(2, T.BIAS, (E, F), 0.3)
    W2 = hapgen.normal(2, T.W2, (E, F, Hd), 0.4); b2 = hapgen.normal(2, T.BETA, (E, Hd), 0.3)
    rows = [6, 0, 3, 5]
    r = layers.moe_ffn_block(X, W1, b1, W2, b2, dOut, rows)
    for e in range(E):
        n = rows[e]
        ref = layers.mlp_block(X[e, :n], W1[e], b1[e], W2[e], b2[e], dOut[e, :n])
        for k in ("pre", "H", "out", "dH", "dX"):
            np.testing.assert_allclose(r[k][e, :n], ref[k], rtol=1e-12, atol=1e-12)
            assert not r[k][e, n:].any()
        for k in ("dW1", "db1", "dW2", "db2"):
            np.testing.assert_allclose(r[k][e], ref[k], rtol=1e-12, atol=1e-12)
    L = lambda X_: float((layers.moe_ffn_block(X_, W1, b1, W2, b2, dOut, rows)["out"] * dOut).sum())
    h = 1e-6
    for idx in [(0, 0, 0), (2, 2, 4), (3, 4, 1), (2, 4, 0)]:
        Xp, Xm = X.copy(), X.copy(); Xp[idx] += h; Xm[idx] -= h
        assert (L(Xp) - L(Xm)) / (2 * h) == pytest.approx(r["dX"][idx], rel=1e-6, abs=1e-7)
