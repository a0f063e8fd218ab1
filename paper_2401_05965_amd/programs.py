"""Per-device instruction sequences of the workloads, as ordered calls into libhap.

A synthesized HAP program is a list of instructions every device executes on its own shard
(Sec. 4.1); the classes here are those lists for the layers the workloads name.  They hold the
device buffers (torch tensors, used as memory only) and call the C ABI; no arithmetic is done
in Python.  `timer`, when given, is called as timer(label, fn) around each library call so a
benchmark can bracket individual launches with events.
"""
from __future__ import annotations

import torch

from . import binding as hap


def _pad8(n: int) -> int:
    return (n + 7) // 8 * 8


def _call(timer, label, fn):
    if timer is None:
        fn()
    else:
        timer(label, fn)


class MlpShard:
    """Device j's share of  H = gelu(X W1 + b1);  Out = H W2  with the ffn axis sharded.

    fc1 follows the feature rule (columns c_j of W1), fc2 the reduction rule (rows c_j of W2): the
    device's output P_j is a partial sum to be all-reduced (bias b2 is added after that, not here).
    Weights are the device's compact slices, as a worker keeps them (Sec. 6), with the leading
    dimension of W1_j rounded up to a multiple of 8 elements.
    """

    def __init__(self, tokens, hidden, ffn, offsets, j, X, W1, b1, W2, dOut, dtype=torch.bfloat16):
        self.T, self.h, self.F, self.j = tokens, hidden, ffn, j
        lo, hi = offsets[j], offsets[j + 1]
        self.f = f = hi - lo
        self.ld = ld = max(_pad8(f), 8)
        dev = X.device
        self.X, self.dOut = X, dOut
        self.W1 = torch.zeros((hidden, ld), dtype=dtype, device=dev); self.W1[:, :f] = W1[:, lo:hi]
        self.b1 = b1[lo:hi].clone() if f else torch.zeros((8,), dtype=dtype, device=dev)
        self.W2 = W2[lo:hi].clone() if f else torch.zeros((8, hidden), dtype=dtype, device=dev)
        self.H = torch.zeros((tokens, ld), dtype=dtype, device=dev)
        self.pre = torch.zeros((tokens, ld), dtype=dtype, device=dev)
        self.P = torch.zeros((tokens, hidden), dtype=dtype, device=dev)
        self.dH = torch.zeros((tokens, ld), dtype=dtype, device=dev)
        self.dX = torch.zeros((tokens, hidden), dtype=dtype, device=dev)
        self.dW1 = torch.zeros((hidden, ld), dtype=dtype, device=dev)
        self.dW2 = torch.zeros((max(f, 1), hidden), dtype=dtype, device=dev)
        self.db1 = torch.zeros((max(f, 1),), dtype=torch.float32, device=dev)
        io = hap.BF16 if dtype == torch.bfloat16 else hap.F32
        self.io = io
        self.fc1 = hap.LinearDesc(tokens, hidden, ffn, hap.SHARD_FEATURE, offsets, io, act=hap.ACT_GELU_ERF, has_bias=True,
                                  ldx=hidden, ldw=ld, ldy=ld, operands_are_full=False)
        self.fc2 = hap.LinearDesc(tokens, ffn, hidden, hap.SHARD_REDUCTION, offsets, io, ldx=ld, ldw=hidden, ldy=hidden,
                                  operands_are_full=False)
        nws = max(hap.hap_linear_bwd_workspace(self.fc1, j), hap.hap_linear_bwd_workspace(self.fc2, j), 256)
        self.ws = torch.empty((nws,), dtype=torch.uint8, device=dev)

    def flops(self):
        """Algorithmic flops of (fwd, bwd): 2 GEMMs forward, 4 backward, 2*M*N*K each."""
        g = 2.0 * self.T * self.h * self.f
        return 2 * g, 4 * g

    def forward(self, timer=None):
        j = self.j
        _call(timer, "fc1_fwd", lambda: hap.hap_sharded_linear_fwd(self.fc1, j, self.X, self.W1, self.b1, self.H, self.pre))
        _call(timer, "fc2_fwd", lambda: hap.hap_sharded_linear_fwd(self.fc2, j, self.H, self.W2, None, self.P, None))

    def backward(self, timer=None):
        j = self.j
        # fc2 (reduction rule): dH_j = dOut W2[c_j,:]^T, dW2[c_j,:] = H_j^T dOut
        _call(timer, "fc2_bwd", lambda: hap.hap_sharded_linear_bwd(self.fc2, j, self.H, self.W2, None, self.dOut, self.dH, self.dW2,
                                                                   self.io, None, self.ws))
        # fc1 (feature rule): dP = dH_j * gelu'(pre_j); dX_j = dP W1_j^T (partial), dW1_j = X^T dP, db1_j = colsum(dP)
        _call(timer, "fc1_bwd", lambda: hap.hap_sharded_linear_bwd(self.fc1, j, self.X, self.W1, self.pre, self.dH, self.dX, self.dW1,
                                                                   self.io, self.db1, self.ws))


class SfbRebuild:
    """dW = sum_i X_i^T dY_i over m devices' gathered factors held in padded-capacity buffers."""

    def __init__(self, Xs, dYs, rows, in_features, out_features):
        self.Xs, self.dYs, self.rows = Xs, dYs, list(rows)
        self.inf, self.outf = in_features, out_features
        self.dW = torch.zeros((in_features, out_features), dtype=torch.float32, device=Xs[0].device)
        self.dtype = hap.BF16 if Xs[0].dtype == torch.bfloat16 else hap.F32

    def flops(self):
        return 2.0 * self.inf * self.outf * sum(self.rows)

    def run(self, timer=None):
        _call(timer, "sfb_grad", lambda: hap.hap_sfb_grad(self.Xs, self.dYs, self.rows, self.inf, self.outf, self.Xs[0].stride(0),
                                                          self.dYs[0].stride(0), self.dtype, self.dW, self.outf))
