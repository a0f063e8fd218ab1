"""Expert-sharded Mixture-of-Experts layer (Sec. 7.6, "Case Study: Uneven Placement of Experts").

An MoE layer holds E experts, each a fully-connected layer of its own: expert e maps the tokens that
were dispatched to it, X_e[C x in] (C = the per-expert buffer capacity, of which the first rows[e]
rows hold tokens), through its own W_e[in x out] and b_e[out].  Expert parallelism shards the EXPERT
axis: device j owns the experts [offsets[j], offsets[j+1]) - any integer split, even or not - and
runs exactly those experts' layers on exactly their tokens.  Nothing is padded: a device with fewer
experts does proportionally less work, and the concatenation of the devices' results over the
expert axis is the unsharded layer (the distributed program reproduces the single-device one).

    Y_e  = act(X_e W_e + b_e)              rows < rows[e]
    dP_e = dY_e * act'(X_e W_e + b_e)
    dX_e = dP_e W_e^T,   dW_e = X_e^T dP_e,   db_e = column sums of dP_e     (over rows < rows[e])

Rows at or beyond rows[e] hold no token: they are never read, and the corresponding output rows are
returned as zeros here (the device library leaves them untouched; tests compare valid rows only).
"""
from __future__ import annotations

import numpy as np

from .pointwise import gelu, gelu_grad


def _f64(a):
    return None if a is None else np.asarray(a, dtype=np.float64)


def _rows(rows, E, C):
    r = np.full(E, C, dtype=np.int64) if rows is None else np.asarray(rows, dtype=np.int64)
    if r.shape != (E,) or (r < 0).any() or (r > C).any():
        raise ValueError("rows must hold one count in [0, capacity] per expert")
    return r


def moe_linear_fwd(X, W, bias=None, rows=None, act=False):
    """All E experts.  X [E x C x in], W [E x in x out], bias [E x out] or None.  Returns (Y, preact) [E x C x out]."""
    X, W, bias = _f64(X), _f64(W), _f64(bias)
    E, C, _ = X.shape
    n = _rows(rows, E, C)
    Y = np.zeros((E, C, W.shape[2])); pre = np.zeros_like(Y)
    for e in range(E):
        p = X[e, :n[e]] @ W[e]
        if bias is not None:
            p = p + bias[e]
        pre[e, :n[e]] = p
        Y[e, :n[e]] = gelu(p) if act else p
    return Y, pre


def moe_linear_bwd(X, W, preact, dY, rows=None, act=False):
    """All E experts.  Returns (dX [E x C x in], dW [E x in x out], db [E x out])."""
    X, W, dY = _f64(X), _f64(W), _f64(dY)
    E, C, _ = X.shape
    n = _rows(rows, E, C)
    dX = np.zeros_like(X); dW = np.zeros_like(W); db = np.zeros((E, W.shape[2]))
    for e in range(E):
        dP = dY[e, :n[e]]
        if act:
            dP = dP * gelu_grad(_f64(preact)[e, :n[e]])
        dX[e, :n[e]] = dP @ W[e].T
        dW[e] = X[e, :n[e]].T @ dP
        db[e] = dP.sum(axis=0)
    return dX, dW, db


def sharded_moe_linear_fwd(offsets, j, X, W, bias=None, rows=None, act=False):
    """Device j's experts [offsets[j], offsets[j+1]) of the unsharded result: (Y_j, preact_j)."""
    Y, pre = moe_linear_fwd(X, W, bias, rows, act)
    s = slice(int(offsets[j]), int(offsets[j + 1]))
    return Y[s], pre[s]


def sharded_moe_linear_bwd(offsets, j, X, W, preact, dY, rows=None, act=False):
    """Device j's experts of (dX, dW, db): exact slices over the expert axis, no partial sums."""
    dX, dW, db = moe_linear_bwd(X, W, preact, dY, rows, act)
    s = slice(int(offsets[j]), int(offsets[j + 1]))
    return dX[s], dW[s], db[s]
