"""Softmax attention on a head or batch slice.

The paper takes Transformer layers as given operators; the definition is the
standard one: per (batch, head), S = Q K^T / sqrt(d), P = softmax over keys,
O = P V; no mask, no dropout.  Heads and batch entries are independent, so a
device's slice is the same computation restricted to its heads / samples.
Tensors are [batch, heads, seq, head_dim].
"""
from __future__ import annotations

import numpy as np


def attn_fwd(Q, K, V):
    """Returns (O, lse) with lse = log sum_k exp(S) per query row."""
    Q, K, V = (np.asarray(t, dtype=np.float64) for t in (Q, K, V))
    scale = 1.0 / np.sqrt(Q.shape[-1])
    S = (Q @ K.swapaxes(-1, -2)) * scale          # [b, h, query, key]; matmul acts on the last two axes
    mx = S.max(axis=-1, keepdims=True)
    E = np.exp(S - mx)
    den = E.sum(axis=-1, keepdims=True)
    P = E / den
    O = P @ V
    return O, (mx + np.log(den))[..., 0]


def attn_bwd(Q, K, V, dO):
    """Returns (dQ, dK, dV)."""
    Q, K, V, dO = (np.asarray(t, dtype=np.float64) for t in (Q, K, V, dO))
    scale = 1.0 / np.sqrt(Q.shape[-1])
    S = (Q @ K.swapaxes(-1, -2)) * scale
    E = np.exp(S - S.max(axis=-1, keepdims=True))
    P = E / E.sum(axis=-1, keepdims=True)
    dV = P.swapaxes(-1, -2) @ dO
    dP = dO @ V.swapaxes(-1, -2)
    dS = P * (dP - (dP * P).sum(axis=-1, keepdims=True))
    dQ = (dS @ K) * scale
    dK = (dS.swapaxes(-1, -2) @ Q) * scale
    return dQ, dK, dV


def slice_heads_or_batch(T, over_heads, offsets, j):
    lo, hi = int(offsets[j]), int(offsets[j + 1])
    return T[:, lo:hi] if over_heads else T[lo:hi]
