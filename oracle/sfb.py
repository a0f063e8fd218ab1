"""Sufficient-factor gradient rebuild (Sec. 2.3.2, Fig. "sfb"(c); replicated MatMul rule of Sec. 4.3).

Every device holds the gathered factors of all m devices - activations
X_i[b_i x in] and output gradients dY_i[b_i x out] - and rebuilds the whole
weight gradient itself:  dW = sum_i X_i^T dY_i, which equals what an
All-Reduce of the per-device local gradients would deliver (Fig. "sfb"(b)).
Buffers may have more rows than b_i (the padded All-Gather layout); rows at or
beyond b_i are not part of the factor and are never read.
"""
from __future__ import annotations

import numpy as np


def sfb_grad(Xs, dYs, rows):
    in_f, out_f = Xs[0].shape[1], dYs[0].shape[1]
    dW = np.zeros((in_f, out_f), dtype=np.float64)
    for X, dY, b in zip(Xs, dYs, rows):
        b = int(b)
        if b:
            dW += np.asarray(X[:b], dtype=np.float64).T @ np.asarray(dY[:b], dtype=np.float64)
    return dW
