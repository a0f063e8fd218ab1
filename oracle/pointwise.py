"""Row-wise and element-wise layer pieces the workloads name (GeLU, LayerNorm).

The paper treats these as given single-device operators; definitions are the
textbook ones: erf-form GeLU, LayerNorm with biased variance over the hidden
axis and eps = 1e-5.
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf

LN_EPS = 1e-5


def gelu(x):
    return 0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))


def gelu_grad(x):
    """d gelu / dx = Phi(x) + x * phi(x)."""
    return 0.5 * (1.0 + erf(x / np.sqrt(2.0))) + x * np.exp(-0.5 * x * x) / np.sqrt(2.0 * np.pi)


def layernorm_fwd(x, gamma, beta, eps=LN_EPS):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    return (x - mu) * rstd * gamma + beta, mu[..., 0], rstd[..., 0]


def layernorm_bwd(x, gamma, dy, eps=LN_EPS):
    """Returns dx, dgamma, dbeta for y = (x-mu)*rstd*gamma + beta."""
    n = x.shape[-1]
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    g = dy * gamma
    dx = rstd * (g - g.mean(axis=-1, keepdims=True) - xhat * (g * xhat).mean(axis=-1, keepdims=True))
    flat_dy = dy.reshape(-1, n)
    dgamma = (flat_dy * xhat.reshape(-1, n)).sum(axis=0)
    dbeta = flat_dy.sum(axis=0)
    return dx, dgamma, dbeta
