"""Pins for oracle.linear and oracle.sfb (Fig. "semantics" MatMul rules; Sec. 2.3.2 / Fig. "sfb")."""
import numpy as np
import pytest

import hapgen
from oracle import linear, sfb, pointwise
from oracle.linear import BATCH, FEATURE, REDUCTION, REPLICATED


def _data(T=13, I=9, O=11, seed=3):
    X = hapgen.normal(seed, hapgen.TensorId.X, (T, I))
    W = hapgen.normal(seed, hapgen.TensorId.W, (I, O), 0.3)
    b = hapgen.normal(seed, hapgen.TensorId.BIAS, (O,), 0.5)
    dY = hapgen.normal(seed, hapgen.TensorId.DY, (T, O))
    return X, W, b, dY


def test_brute_force_three_loops_exact_on_integers():
    rng = np.random.default_rng(0)
    X = rng.integers(-4, 5, (5, 6)).astype(float); W = rng.integers(-4, 5, (6, 7)).astype(float)
    b = rng.integers(-4, 5, 7).astype(float); dY = rng.integers(-4, 5, (5, 7)).astype(float)
    Y, pre = linear.linear_fwd(X, W, b)
    dX, dW, db = linear.linear_bwd(X, W, pre, dY)
    for t in range(5):
        for o in range(7):
            assert Y[t, o] == sum(X[t, i] * W[i, o] for i in range(6)) + b[o]
    for t in range(5):
        for i in range(6):
            assert dX[t, i] == sum(dY[t, o] * W[i, o] for o in range(7))
    for i in range(6):
        for o in range(7):
            assert dW[i, o] == sum(X[t, i] * dY[t, o] for t in range(5))
    for o in range(7):
        assert db[o] == sum(dY[t, o] for t in range(5))


def test_identity_and_one_hot():
    X, W, b, dY = _data(I=9, O=9)
    Y, _ = linear.linear_fwd(X, np.eye(9))
    assert np.array_equal(Y, X)
    onehot = np.zeros((3, 9)); onehot[0, 4] = onehot[1, 0] = onehot[2, 8] = 1
    Y, _ = linear.linear_fwd(onehot, W)
    assert np.array_equal(Y, W[[4, 0, 8]])


@pytest.mark.parametrize("act", [False, True])
def test_finite_differences(act):
    X, W, b, dY = _data()
    Y, pre = linear.linear_fwd(X, W, b, act)
    dX, dW, db = linear.linear_bwd(X, W, pre, dY, act)
    L = lambda X_, W_, b_: float((linear.linear_fwd(X_, W_, b_, act)[0] * dY).sum())
    h = 1e-6
    for (t, i) in [(0, 0), (5, 3), (12, 8)]:
        Xp, Xm = X.copy(), X.copy(); Xp[t, i] += h; Xm[t, i] -= h
        assert (L(Xp, W, b) - L(Xm, W, b)) / (2 * h) == pytest.approx(dX[t, i], rel=1e-6, abs=1e-7)
    for (i, o) in [(0, 0), (4, 10), (8, 5)]:
        Wp, Wm = W.copy(), W.copy(); Wp[i, o] += h; Wm[i, o] -= h
        assert (L(X, Wp, b) - L(X, Wm, b)) / (2 * h) == pytest.approx(dW[i, o], rel=1e-6, abs=1e-7)
    for o in [0, 6, 10]:
        bp, bm = b.copy(), b.copy(); bp[o] += h; bm[o] -= h
        assert (L(X, W, bp) - L(X, W, bm)) / (2 * h) == pytest.approx(db[o], rel=1e-6, abs=1e-7)


@pytest.mark.parametrize("act", [False, True])
def test_shards_concatenate_or_sum_to_unsharded(act):
    X, W, b, dY = _data()
    Y, pre = linear.linear_fwd(X, W, b, act)
    dX, dW, db = linear.linear_bwd(X, W, pre, dY, act)
    # batch rule: rows concatenate; weight/bias gradients are partials
    offs = [0, 6, 6, 10, 13]
    parts = [linear.sharded_linear_fwd(BATCH, offs, j, X, W, b, act)[0] for j in range(4)]
    assert np.allclose(np.concatenate(parts, 0), Y, rtol=0, atol=1e-13)
    g = [linear.sharded_linear_bwd(BATCH, offs, j, X, W, pre, dY, act) for j in range(4)]
    assert np.allclose(np.concatenate([x[0] for x in g], 0), dX, atol=1e-12)
    assert np.allclose(sum(x[1] for x in g), dW, atol=1e-12)
    assert np.allclose(sum(x[2] for x in g), db, atol=1e-12)
    # feature rule: columns concatenate; dX is a partial
    offs = [0, 5, 7, 11]
    parts = [linear.sharded_linear_fwd(FEATURE, offs, j, X, W, b, act)[0] for j in range(3)]
    assert np.allclose(np.concatenate(parts, 1), Y, atol=1e-13)
    g = [linear.sharded_linear_bwd(FEATURE, offs, j, X, W, pre, dY, act) for j in range(3)]
    assert np.allclose(sum(x[0] for x in g), dX, atol=1e-12)
    assert np.allclose(np.concatenate([x[1] for x in g], 1), dW, atol=1e-12)
    assert np.allclose(np.concatenate([x[2] for x in g]), db, atol=1e-12)
    if not act:
        # reduction rule: partial products sum (the All-Reduce), gradients slice
        offs = [0, 2, 9]
        Y0, pre0 = linear.linear_fwd(X, W)
        parts = [linear.sharded_linear_fwd(REDUCTION, offs, j, X, W)[0] for j in range(2)]
        assert np.allclose(sum(parts), Y0, atol=1e-12)
        g = [linear.sharded_linear_bwd(REDUCTION, offs, j, X, W, None, dY) for j in range(2)]
        dX0, dW0, _ = linear.linear_bwd(X, W, pre0, dY)
        assert np.allclose(np.concatenate([x[0] for x in g], 1), dX0, atol=1e-12)
        assert np.allclose(np.concatenate([x[1] for x in g], 0), dW0, atol=1e-12)
        with pytest.raises(ValueError):
            linear.sharded_linear_fwd(REDUCTION, offs, 0, X, W, b)
    # replicated rule
    assert np.array_equal(linear.sharded_linear_fwd(REPLICATED, [0, 13], 0, X, W, b, act)[0], Y)


# ---------------- SFB ----------------

def _factors(rows, cap, I=7, O=5, seed=1):
    Xs = [hapgen.normal(seed, hapgen.TensorId.SFB_X + i, (cap, I)) for i in range(len(rows))]
    dYs = [hapgen.normal(seed, hapgen.TensorId.SFB_DY + i, (cap, O)) for i in range(len(rows))]
    return Xs, dYs


def test_sfb_equals_all_reduced_local_gradients_and_unsharded():
    rows = [6, 0, 3, 8, 1]
    Xs, dYs = _factors(rows, 8)
    got = sfb.sfb_grad(Xs, dYs, rows)
    naive = sum(linear.linear_bwd(X[:b], np.zeros((7, 5)), None, dY[:b])[1] for X, dY, b in zip(Xs, dYs, rows))
    assert np.allclose(got, naive, atol=1e-12)
    Xc = np.concatenate([X[:b] for X, b in zip(Xs, rows)]); dYc = np.concatenate([d[:b] for d, b in zip(dYs, rows)])
    assert np.allclose(got, Xc.T @ dYc, atol=1e-12)
    # brute force
    ref = np.zeros((7, 5))
    for X, dY, b in zip(Xs, dYs, rows):
        for r in range(b):
            for i in range(7):
                for o in range(5):
                    ref[i, o] += X[r, i] * dY[r, o]
    assert np.allclose(got, ref, atol=1e-12)


def test_sfb_never_reads_padding_rows_and_degenerate_cases():
    rows = [2, 5, 0]
    Xs, dYs = _factors(rows, 6)
    clean = sfb.sfb_grad(Xs, dYs, rows)
    for X, dY, b in zip(Xs, dYs, rows):
        X[b:] = np.nan; dY[b:] = np.nan
    assert np.array_equal(sfb.sfb_grad(Xs, dYs, rows), clean) and np.isfinite(clean).all()
    assert np.array_equal(sfb.sfb_grad(Xs[:1], dYs[:1], [2]), Xs[0][:2].T @ dYs[0][:2])
    assert np.array_equal(sfb.sfb_grad(Xs, dYs, [0, 0, 0]), np.zeros((7, 5)))


def test_sfb_gradient_is_low_rank_when_global_batch_is_small():
    # Sec. 2.3.2: with total batch B below both matrix dimensions the gradient has rank <= B
    rows = [2, 1]
    Xs, dYs = _factors(rows, 2, I=12, O=10)
    assert np.linalg.matrix_rank(sfb.sfb_grad(Xs, dYs, rows)) == 3
