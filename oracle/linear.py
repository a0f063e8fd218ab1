"""Sharded fully-connected layer (Fig. "semantics": the three MatMul sharding rules,
plus the replicated rule added for sufficient-factor broadcasting in Sec. 4.3).

Conventions: X[tokens x in], W[in x out], Y = act(X W + b); dX = dP W^T,
dW = X^T dP, db = column sums of dP, with dP = dY * act'(X W + b).

The distributed program must reproduce the single-device result, so each
function evaluates the unsharded definition on the full tensors and then takes
device j's slice [offsets[j], offsets[j+1]) of the sharded axis; a
reduction-sharded product is device j's partial sum over its slice of the
contracted axis, whose sum over devices is the unsharded result.
"""
from __future__ import annotations

import numpy as np

from .pointwise import gelu, gelu_grad

BATCH, FEATURE, REDUCTION, REPLICATED = 0, 1, 2, 3


def _f64(a):
    return None if a is None else np.asarray(a, dtype=np.float64)


def _rng(offsets, j):
    return slice(int(offsets[j]), int(offsets[j + 1]))


def linear_fwd(X, W, bias=None, act=False):
    """Unsharded layer. Returns (Y, preact)."""
    X, W, bias = _f64(X), _f64(W), _f64(bias)
    pre = X @ W
    if bias is not None:
        pre = pre + bias
    return (gelu(pre) if act else pre), pre


def linear_bwd(X, W, preact, dY, act=False):
    """Unsharded backward. Returns (dX, dW, db)."""
    X, W, dY = _f64(X), _f64(W), _f64(dY)
    dP = dY * gelu_grad(_f64(preact)) if act else dY
    return dP @ W.T, X.T @ dP, dP.sum(axis=0)


def sharded_linear_fwd(mode, offsets, j, X, W, bias=None, act=False):
    """Device j's output for the given rule.  Returns (Y_j, preact_j).

    BATCH:     rows r_j of Y            (e1|AG(0), e2|Id  -> e3|AG(0))
    FEATURE:   columns c_j of Y         (e1|Id, e2|AG(1)  -> e3|AG(1))
    REDUCTION: partial X[:,k_j] W[k_j,:] (e1|AG(1), e2|AG(0) -> e3|All-Reduce); no bias, no activation
    """
    X, W, bias = _f64(X), _f64(W), _f64(bias)
    if mode == REDUCTION:
        if bias is not None or act:
            raise ValueError("bias/activation apply after the all-reduce, not to a partial")
        k = _rng(offsets, j)
        P = X[:, k] @ W[k, :]
        return P, P
    Y, pre = linear_fwd(X, W, bias, act)
    if mode == BATCH:
        r = _rng(offsets, j)
        return Y[r, :], pre[r, :]
    if mode == FEATURE:
        c = _rng(offsets, j)
        return Y[:, c], pre[:, c]
    return Y, pre


def sharded_linear_bwd(mode, offsets, j, X, W, preact, dY, act=False):
    """Device j's (dX_j, dW_j, db_j) given full-size X, W, preact, dY.

    BATCH:     dX rows r_j (exact slice); dW_j, db_j are partials over the device's rows (sum over j = full)
    FEATURE:   dX_j is a partial (sum over j = full); dW, db columns c_j (exact slices)
    REDUCTION: dX columns k_j, dW rows k_j (exact slices); db not defined (None)
    """
    X, W, dY = _f64(X), _f64(W), _f64(dY)
    if mode == REDUCTION:
        if act:
            raise ValueError("no activation on a partial")
        k = _rng(offsets, j)
        return dY @ W[k, :].T, X[:, k].T @ dY, None
    dP = dY * gelu_grad(_f64(preact)) if act else dY
    if mode == BATCH:
        r = _rng(offsets, j)
        return dP[r, :] @ W.T, X[r, :].T @ dP[r, :], dP[r, :].sum(axis=0)
    if mode == FEATURE:
        c = _rng(offsets, j)
        return dP[:, c] @ W[:, c].T, X.T @ dP[:, c], dP[:, c].sum(axis=0)
    return dP @ W.T, X.T @ dP, dP.sum(axis=0)
