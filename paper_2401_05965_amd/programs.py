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


def _pitch(n: int) -> int:
    """Leading dimension (bf16 elements) of a device's compact slice of width n: the next multiple of 64 elements = 128 bytes.
    Rows that start on a 128-byte boundary keep the row fetches of K-contiguous GEMM operands inside one cache sector each
    (with a pitch of only 8 elements every fetch straddles two: 10-20 % of a product's time, measured)."""
    return max((n + 63) // 64 * 64, 64)


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
    dimension of W1_j rounded up to a multiple of 64 elements (128 bytes).
    """

    def __init__(self, tokens, hidden, ffn, offsets, j, X, W1, b1, W2, dOut, dtype=torch.bfloat16, whole_tensors=False, fuse_act_bwd=None):
        self.T, self.h, self.F, self.j = tokens, hidden, ffn, j
        # fuse_act_bwd: fc2's backward multiplies its dX product by gelu'(pre) in the epilogue, so the buffer `dH` receives
        # dP = dH * gelu'(pre) directly (`dH_holds` names which of the two it holds) and fc1's backward skips that pass.
        # Default on: measured -3 % of the backward for compact slices, -1 % for whole tensors.
        if fuse_act_bwd is None:
            fuse_act_bwd = True
        self.fuse_act_bwd = fuse_act_bwd
        self.dH_holds = "dP" if fuse_act_bwd else "dH"
        lo, hi = offsets[j], offsets[j + 1]
        self.f = f = hi - lo
        dev = X.device
        self.X, self.dOut = X, dOut
        io = hap.BF16 if dtype == torch.bfloat16 else hap.F32
        self.io = io
        if whole_tensors:
            # The other way to hand a shard to the library (operands_are_full = 1): every tensor is passed whole and the library
            # applies the device's range [lo, hi) itself - zero-copy views that start at arbitrary elements.  Results land in the
            # device's columns / rows of whole-size buffers; `cols` is that range.
            self.ld = ld = ffn
            self.cols = slice(lo, hi)
            self.W1, self.b1, self.W2 = W1, b1, W2
            z = lambda *shape, dt=dtype: torch.zeros(shape, dtype=dt, device=dev)
            self.H, self.pre, self.dH = z(tokens, ffn), z(tokens, ffn), z(tokens, ffn)
            self.P, self.dX = z(tokens, hidden), z(tokens, hidden)
            self.dW1, self.dW2, self.db1 = z(hidden, ffn), z(ffn, hidden), z(ffn, dt=torch.float32)
            self.fc1 = hap.LinearDesc(tokens, hidden, ffn, hap.SHARD_FEATURE, offsets, io, act=hap.ACT_GELU_ERF, has_bias=True,
                                      ldx=hidden, ldw=ffn, ldy=ffn, operands_are_full=True)
            self.fc2 = hap.LinearDesc(tokens, ffn, hidden, hap.SHARD_REDUCTION, offsets, io, ldx=ffn, ldw=hidden, ldy=hidden,
                                      operands_are_full=True)
            self.fc1_lin = hap.LinearDesc(tokens, hidden, ffn, hap.SHARD_FEATURE, offsets, io, has_bias=True,
                                          ldx=hidden, ldw=ffn, ldy=ffn, operands_are_full=True)
            nws = max(hap.hap_linear_bwd_workspace(self.fc1, j), hap.hap_linear_bwd_workspace(self.fc2, j), 256)
            self.ws = torch.empty((nws,), dtype=torch.uint8, device=dev)
            return
        self.ld = ld = _pitch(f)
        self.cols = slice(0, f)
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
        self.fc1 = hap.LinearDesc(tokens, hidden, ffn, hap.SHARD_FEATURE, offsets, io, act=hap.ACT_GELU_ERF, has_bias=True,
                                  ldx=hidden, ldw=ld, ldy=ld, operands_are_full=False)
        self.fc2 = hap.LinearDesc(tokens, ffn, hidden, hap.SHARD_REDUCTION, offsets, io, ldx=ld, ldw=hidden, ldy=hidden,
                                  operands_are_full=False)
        self.fc1_lin = hap.LinearDesc(tokens, hidden, ffn, hap.SHARD_FEATURE, offsets, io, has_bias=True,
                                      ldx=hidden, ldw=ld, ldy=ld, operands_are_full=False)    # fc1 with its activation already differentiated
        nws = max(hap.hap_linear_bwd_workspace(self.fc1, j), hap.hap_linear_bwd_workspace(self.fc2, j), 256)
        self.ws = torch.empty((nws,), dtype=torch.uint8, device=dev)      # also serves the forward's optional split-K scratch

    def flops(self):
        """Algorithmic flops of (fwd, bwd): 2 GEMMs forward, 4 backward, 2*M*N*K each."""
        g = 2.0 * self.T * self.h * self.f
        return 2 * g, 4 * g

    def forward(self, timer=None):
        j = self.j
        _call(timer, "fc1_fwd", lambda: hap.hap_sharded_linear_fwd(self.fc1, j, self.X, self.W1, self.b1, self.H, self.pre, self.ws))
        _call(timer, "fc2_fwd", lambda: hap.hap_sharded_linear_fwd(self.fc2, j, self.H, self.W2, None, self.P, None, self.ws))

    def backward(self, timer=None):
        j = self.j
        if self.fuse_act_bwd:
            # fc2 (reduction rule): dP_j = (dOut W2[c_j,:]^T) * gelu'(pre_j) in one product, dW2[c_j,:] = H_j^T dOut
            _call(timer, "fc2_bwd", lambda: hap.hap_sharded_linear_bwd_dact(self.fc2, j, self.H, self.W2, None, self.dOut, self.dH, self.dW2,
                                                                            self.io, None, self.pre, hap.ACT_GELU_ERF, self.ws))
            # fc1 (feature rule) on dP: dX_j = dP W1_j^T (partial), dW1_j = X^T dP, db1_j = colsum(dP)
            _call(timer, "fc1_bwd", lambda: hap.hap_sharded_linear_bwd(self.fc1_lin, j, self.X, self.W1, None, self.dH, self.dX, self.dW1,
                                                                       self.io, self.db1, self.ws))
            return
        # fc2 (reduction rule): dH_j = dOut W2[c_j,:]^T, dW2[c_j,:] = H_j^T dOut
        _call(timer, "fc2_bwd", lambda: hap.hap_sharded_linear_bwd(self.fc2, j, self.H, self.W2, None, self.dOut, self.dH, self.dW2,
                                                                   self.io, None, self.ws))
        # fc1 (feature rule): dP = dH_j * gelu'(pre_j); dX_j = dP W1_j^T (partial), dW1_j = X^T dP, db1_j = colsum(dP)
        _call(timer, "fc1_bwd", lambda: hap.hap_sharded_linear_bwd(self.fc1, j, self.X, self.W1, self.pre, self.dH, self.dX, self.dW1,
                                                                   self.io, self.db1, self.ws))



class MoeExpertShard:
    """Device j's experts of an MoE feed-forward layer (Sec. 7.6): for each expert e the device owns,

        H_e = gelu(X_e W1_e + b1_e);   Out_e = H_e W2_e + b2_e        on the rows[e] tokens dispatched to e

    Expert parallelism shards the expert axis, so nothing is summed across devices: the device's
    outputs and gradients are exact slices.  Buffers are the device's compact [experts_j x ...] slices;
    `rows` (int32, on the device) holds the token count of every expert buffer.
    """

    def __init__(self, experts, capacity, hidden, ffn, offsets, j, X, W1, b1, W2, b2, rows, dOut, dtype=torch.bfloat16, fuse_act_bwd=True):
        self.j, self.C, self.h, self.f = j, capacity, hidden, ffn
        # fuse_act_bwd: fc2's backward multiplies its dX products by gelu'(pre) in the epilogue; `dH` then holds dP (see MlpShard)
        self.fuse_act_bwd = fuse_act_bwd
        self.dH_holds = "dP" if fuse_act_bwd else "dH"
        lo, hi = offsets[j], offsets[j + 1]
        self.n = n = hi - lo
        dev = X.device
        io = self.io = hap.BF16 if dtype == torch.bfloat16 else hap.F32
        sl = slice(lo, hi)
        self.X, self.dOut = X[sl].contiguous(), dOut[sl].contiguous()
        self.W1, self.b1, self.W2, self.b2 = W1[sl].contiguous(), b1[sl].contiguous(), W2[sl].contiguous(), b2[sl].contiguous()
        self.rows = rows[sl].contiguous() if rows is not None else None
        z = lambda *shape: torch.zeros(shape, dtype=dtype, device=dev)
        m = max(n, 1)
        self.H, self.pre, self.dH = z(m, capacity, ffn), z(m, capacity, ffn), z(m, capacity, ffn)
        self.Out, self.dX = z(m, capacity, hidden), z(m, capacity, hidden)
        self.dW1, self.dW2 = z(m, hidden, ffn), z(m, ffn, hidden)
        self.db1 = torch.zeros((m, ffn), dtype=torch.float32, device=dev)
        self.db2 = torch.zeros((m, hidden), dtype=torch.float32, device=dev)
        self.fc1 = hap.MoeDesc(experts, capacity, hidden, ffn, offsets, io, act=hap.ACT_GELU_ERF, has_bias=True, operands_are_full=False)
        self.fc2 = hap.MoeDesc(experts, capacity, ffn, hidden, offsets, io, has_bias=True, operands_are_full=False)
        self.fc1_lin = hap.MoeDesc(experts, capacity, hidden, ffn, offsets, io, has_bias=True, operands_are_full=False)
        nws = max(hap.hap_moe_linear_bwd_workspace(self.fc1, j), hap.hap_moe_linear_bwd_workspace(self.fc2, j), 256)
        self.ws = torch.empty((nws,), dtype=torch.uint8, device=dev)

    def flops(self, rows_host=None):
        """Algorithmic flops of (fwd, bwd) over the tokens actually held: 2 GEMMs forward, 4 backward, 2*M*N*K each."""
        tokens = float(sum(rows_host)) if rows_host is not None else float(self.n * self.C)
        g = 2.0 * tokens * self.h * self.f
        return 2 * g, 4 * g

    def forward(self, timer=None):
        j = self.j
        _call(timer, "moe_fc1_fwd", lambda: hap.hap_moe_linear_fwd(self.fc1, j, self.X, self.W1, self.b1, self.rows, self.H, self.pre, self.ws))
        _call(timer, "moe_fc2_fwd", lambda: hap.hap_moe_linear_fwd(self.fc2, j, self.H, self.W2, self.b2, self.rows, self.Out, None, self.ws))

    def backward(self, timer=None):
        j = self.j
        if self.fuse_act_bwd:
            _call(timer, "moe_fc2_bwd", lambda: hap.hap_moe_linear_bwd_dact(self.fc2, j, self.H, self.W2, None, self.dOut, self.rows, self.dH, self.dW2,
                                                                            self.io, self.db2, self.pre, hap.ACT_GELU_ERF, self.ws))
            _call(timer, "moe_fc1_bwd", lambda: hap.hap_moe_linear_bwd(self.fc1_lin, j, self.X, self.W1, None, self.dH, self.rows, self.dX, self.dW1,
                                                                       self.io, self.db1, self.ws))
            return
        _call(timer, "moe_fc2_bwd", lambda: hap.hap_moe_linear_bwd(self.fc2, j, self.H, self.W2, None, self.dOut, self.rows, self.dH, self.dW2,
                                                                   self.io, self.db2, self.ws))
        _call(timer, "moe_fc1_bwd", lambda: hap.hap_moe_linear_bwd(self.fc1, j, self.X, self.W1, self.pre, self.dH, self.rows, self.dX, self.dW1,
                                                                   self.io, self.db1, self.ws))

class SfbRebuild:
    """dW = sum_i X_i^T dY_i over m devices' gathered factors held in padded-capacity buffers."""

    def __init__(self, Xs, dYs, rows, in_features, out_features):
        self.Xs, self.dYs, self.rows = Xs, dYs, list(rows)
        self.inf, self.outf = in_features, out_features
        self.dW = torch.zeros((in_features, out_features), dtype=torch.float32, device=Xs[0].device)
        self.dtype = hap.BF16 if Xs[0].dtype == torch.bfloat16 else hap.F32
        self.ws = torch.empty((hap.hap_sfb_workspace(len(self.rows), self.rows, in_features, out_features),), dtype=torch.uint8, device=Xs[0].device)

    def flops(self):
        return 2.0 * self.inf * self.outf * sum(self.rows)

    def run(self, timer=None):
        _call(timer, "sfb_grad", lambda: hap.hap_sfb_grad(self.Xs, self.dYs, self.rows, self.inf, self.outf, self.Xs[0].stride(0),
                                                          self.dYs[0].stride(0), self.dtype, self.dW, self.outf, ws=self.ws))


def _zeros(shape, dtype, dev):
    return torch.zeros(shape, dtype=dtype, device=dev)


class EncoderShard:
    """Device j's instructions of one pre-LayerNorm Transformer encoder layer.

        x1 = x + Attn(LN1(x)) Wo + bo ;   y = x1 + gelu(LN2(x1) W1 + b1) W2 + b2

    Two sharding styles share the instruction list:
      "tensor": heads and the ffn axis are sharded (feature rule for Wq/Wk/Wv/W1, reduction rule
                for Wo/W2); tokens are whole; the Wo and W2 products are partial sums that the
                caller all-reduces (here: adds up over the virtual devices) before the residual.
      "data":   the batch is sharded (batch rule everywhere); weights are whole; outputs are exact
                row slices and the weight gradients are partial sums over the batch.
    The device keeps its Wq|Wk|Wv slices side by side in one [hidden x 3*heads_j*d] buffer so the
    three projections (and their backward) run as single GEMMs.
    """

    def __init__(self, style, j, B, S, hidden, heads, d, ffn, head_offsets, ffn_offsets, batch_offsets, params, dtype=torch.bfloat16):
        assert style in ("tensor", "data")
        self.style, self.j = style, j
        dev = params["Wq"].device
        self.S, self.hidden, self.d = S, hidden, d
        if style == "tensor":
            h0, h1 = head_offsets[j], head_offsets[j + 1]
            f0, f1 = ffn_offsets[j], ffn_offsets[j + 1]
            self.B, self.b0 = B, 0
        else:
            h0, h1, f0, f1 = 0, heads, 0, ffn
            self.b0 = batch_offsets[j]; self.B = batch_offsets[j + 1] - batch_offsets[j]
        self.nh, self.f = h1 - h0, f1 - f0
        self.hd = hd = self.nh * d
        self.N = N = self.B * S
        self.ldf = ldf = _pitch(self.f)
        io = self.io = hap.BF16
        c0, c1 = h0 * d, h1 * d
        self.Wqkv = torch.cat([params[n][:, c0:c1] for n in ("Wq", "Wk", "Wv")], dim=1).contiguous() if hd else _zeros((hidden, 8), dtype, dev)
        self.bqkv = torch.cat([params[n][c0:c1] for n in ("bq", "bk", "bv")]).contiguous() if hd else _zeros((8,), dtype, dev)
        self.Wo = params["Wo"][c0:c1].contiguous() if hd else _zeros((8, hidden), dtype, dev)
        self.W1 = _zeros((hidden, ldf), dtype, dev); self.W1[:, :self.f] = params["W1"][:, f0:f1]
        self.b1 = params["b1"][f0:f1].contiguous() if self.f else _zeros((8,), dtype, dev)
        self.W2 = params["W2"][f0:f1].contiguous() if self.f else _zeros((8, hidden), dtype, dev)
        self.g1, self.be1, self.g2, self.be2 = params["g1"], params["be1"], params["g2"], params["be2"]
        # activations saved for the backward
        z = lambda *s: _zeros(s, dtype, dev)
        zf = lambda *s: _zeros(s, torch.float32, dev)
        self.ln1, self.ln2 = z(N, hidden), z(N, hidden)
        self.mean1, self.rstd1, self.mean2, self.rstd2 = zf(N), zf(N), zf(N), zf(N)
        self.qkv, self.o = z(N, max(3 * hd, 8)), z(N, max(hd, 8))
        self.lse = zf(self.B, max(self.nh, 1), S)
        self.attn_part, self.mlp_part = z(N, hidden), z(N, hidden)
        self.H, self.pre = z(N, ldf), z(N, ldf)
        # gradients
        self.dH, self.dln2_part, self.dln1_part = z(N, ldf), z(N, hidden), z(N, hidden)
        self.do, self.dqkv = z(N, max(hd, 8)), z(N, max(3 * hd, 8))
        self.dWqkv, self.dWo = z(hidden, max(3 * hd, 8)), z(max(hd, 1), hidden)
        self.dW1, self.dW2 = z(hidden, ldf), z(max(self.f, 1), hidden)
        self.dbqkv, self.db1 = zf(max(3 * hd, 1)), zf(max(self.f, 1))
        self.dg1, self.dbe1, self.dg2, self.dbe2 = zf(hidden), zf(hidden), zf(hidden), zf(hidden)
        L = hap.LinearDesc
        one = [0, 1]
        self.d_qkv = L(N, hidden, max(3 * hd, 1), hap.REPLICATED, one, io, has_bias=True, ldx=hidden, ldw=max(3 * hd, 8), ldy=max(3 * hd, 8), m=1)
        self.d_wo = L(N, max(hd, 1), hidden, hap.REPLICATED, one, io, ldx=max(hd, 8), ldw=hidden, ldy=hidden, m=1)
        self.d_fc1 = L(N, hidden, max(self.f, 1), hap.REPLICATED, one, io, act=hap.ACT_GELU_ERF, has_bias=True, ldx=hidden, ldw=ldf, ldy=ldf, m=1)
        self.d_fc2 = L(N, max(self.f, 1), hidden, hap.REPLICATED, one, io, ldx=ldf, ldw=hidden, ldy=hidden, m=1)
        self.d_fc1_lin = L(N, hidden, max(self.f, 1), hap.REPLICATED, one, io, has_bias=True, ldx=hidden, ldw=ldf, ldy=ldf, m=1)
        # Q|K|V are column blocks of the [N x 3hd] projection output; O and dO are [N x hd]
        self.d_attn = hap.AttnDesc(self.B, max(self.nh, 1), S, d, True, [0, max(self.nh, 1)], stride_b=S * 3 * hd, stride_s=3 * hd, stride_h=d,
                                   o_strides=(S * hd, hd, d)) if hd and self.B else None    # no (batch entry, head) pair: no attention call
        nws = max([hap.hap_linear_bwd_workspace(x, 0) for x in (self.d_qkv, self.d_wo, self.d_fc1, self.d_fc2)] +
                  [hap.hap_layernorm_bwd_workspace(N, hidden), hap.hap_colsum_workspace(N, hidden),
                   hap.hap_attn_bwd_workspace(self.d_attn, 0) if self.d_attn is not None else 0, 256])
        self.ws = torch.empty((nws,), dtype=torch.uint8, device=dev)

    # ---- token rows of this device inside whole [tokens x hidden] tensors
    def rows(self, t):
        return t[self.b0 * self.S:(self.b0 + self.B) * self.S]

    def flops(self):
        """Algorithmic flops (fwd, bwd): GEMMs 2*M*N*K, attention 4*S^2*d per (batch, head); backward = 2x forward."""
        g = 2.0 * self.N * self.hidden * (3 * self.hd) + 2.0 * self.N * self.hd * self.hidden + 4.0 * self.N * self.hidden * self.f
        a = 4.0 * self.B * self.nh * self.S * self.S * self.d
        return g + a, 2 * (g + a)

    def attn_forward(self, x, timer=None):
        """x: this device's token rows [N x hidden].  Leaves the Wo product in attn_part."""
        N, hd, io = self.N, self.hd, self.io
        _call(timer, "ln1_fwd", lambda: hap.hap_layernorm_fwd(N, self.hidden, io, x, self.g1, self.be1, self.ln1, self.mean1, self.rstd1))
        if hd == 0:
            self.attn_part.zero_()
            return
        _call(timer, "qkv_fwd", lambda: hap.hap_sharded_linear_fwd(self.d_qkv, 0, self.ln1, self.Wqkv, self.bqkv, self.qkv, None, self.ws))
        q = self.qkv.data_ptr()
        if self.d_attn is not None:
            _call(timer, "attn_fwd", lambda: hap.hap_sharded_attn_fwd(self.d_attn, 0, q, q + hd * 2, q + 2 * hd * 2, self.o, self.lse))
        _call(timer, "wo_fwd", lambda: hap.hap_sharded_linear_fwd(self.d_wo, 0, self.o, self.Wo, None, self.attn_part, None, self.ws))

    def mlp_forward(self, x1, timer=None):
        N, io = self.N, self.io
        _call(timer, "ln2_fwd", lambda: hap.hap_layernorm_fwd(N, self.hidden, io, x1, self.g2, self.be2, self.ln2, self.mean2, self.rstd2))
        if self.f == 0:
            self.mlp_part.zero_()
            return
        _call(timer, "fc1_fwd", lambda: hap.hap_sharded_linear_fwd(self.d_fc1, 0, self.ln2, self.W1, self.b1, self.H, self.pre, self.ws))
        _call(timer, "fc2_fwd", lambda: hap.hap_sharded_linear_fwd(self.d_fc2, 0, self.H, self.W2, None, self.mlp_part, None, self.ws))

    def mlp_backward(self, dy, timer=None):
        """dy: gradient of the layer output on this device's rows.  Leaves the fc1 bwd-data product in dln2_part."""
        if self.f == 0:
            self.dln2_part.zero_()
            return
        # fc2's backward hands fc1 its dP: the GeLU backward rides in the epilogue of the dH product (dH then holds dP)
        _call(timer, "fc2_bwd", lambda: hap.hap_sharded_linear_bwd_dact(self.d_fc2, 0, self.H, self.W2, None, dy, self.dH, self.dW2, self.io, None,
                                                                        self.pre, hap.ACT_GELU_ERF, self.ws))
        _call(timer, "fc1_bwd", lambda: hap.hap_sharded_linear_bwd(self.d_fc1_lin, 0, self.ln2, self.W1, None, self.dH, self.dln2_part, self.dW1, self.io, self.db1, self.ws))

    def ln2_backward(self, x1, dln2, dres, dx1, timer=None):
        """dx1 = dres + LayerNorm2-backward(dln2): the residual path's gradient joins in the same kernel."""
        _call(timer, "ln2_bwd", lambda: hap.hap_layernorm_bwd(self.N, self.hidden, self.io, x1, self.g2, self.mean2, self.rstd2, dln2, dx1,
                                                              self.dg2, self.dbe2, self.ws, dresidual=dres))

    def attn_backward(self, dx1, timer=None):
        """dx1: gradient at the residual stream after attention.  Leaves the QKV bwd-data product in dln1_part."""
        hd = self.hd
        if hd == 0:
            self.dln1_part.zero_()
            return
        _call(timer, "wo_bwd", lambda: hap.hap_sharded_linear_bwd(self.d_wo, 0, self.o, self.Wo, None, dx1, self.do, self.dWo, self.io, None, self.ws))
        q, dq = self.qkv.data_ptr(), self.dqkv.data_ptr()
        if self.d_attn is not None:
            _call(timer, "attn_bwd", lambda: hap.hap_sharded_attn_bwd(self.d_attn, 0, q, q + hd * 2, q + 2 * hd * 2, self.o, self.lse, self.do,
                                                                      dq, dq + hd * 2, dq + 2 * hd * 2, self.ws))
        _call(timer, "qkv_bwd", lambda: hap.hap_sharded_linear_bwd(self.d_qkv, 0, self.ln1, self.Wqkv, None, self.dqkv, self.dln1_part, self.dWqkv,
                                                                   self.io, self.dbqkv, self.ws))

    def ln1_backward(self, x, dln1, dres, dx, timer=None):
        _call(timer, "ln1_bwd", lambda: hap.hap_layernorm_bwd(self.N, self.hidden, self.io, x, self.g1, self.mean1, self.rstd1, dln1, dx,
                                                              self.dg1, self.dbe1, self.ws, dresidual=dres))

    def device_step(self, x, dy, buf, bo, b2):
        """Every instruction device j runs for one forward + backward of the layer, in order, with its own
        partial products standing in for what the All-Reduce would deliver (timing aid: the values equal the
        layer's only when j is the single device).  buf: dict of [N x hidden] tensors x1, y, dx1, dx and fp32
        [hidden] vectors dbo, db2."""
        N, h = self.N, self.hidden
        add = lambda a, b, bias, out: hap.hap_add(N, h, self.io, a, h, b, h, bias, out, h)
        self.attn_forward(x); add(x, self.attn_part, bo, buf["x1"])
        self.mlp_forward(buf["x1"]); add(buf["x1"], self.mlp_part, b2, buf["y"])
        self.mlp_backward(dy); self.ln2_backward(buf["x1"], self.dln2_part, dy, buf["dx1"])
        self.attn_backward(buf["dx1"]); self.ln1_backward(x, self.dln1_part, buf["dx1"], buf["dx"])
        hap.hap_colsum(N, h, self.io, dy, h, buf["db2"], self.ws)
        hap.hap_colsum(N, h, self.io, buf["dx1"], h, buf["dbo"], self.ws)


class EncoderLayerProgram:
    """All virtual devices' EncoderShards run in turn on the one GPU.

    What a cluster would do with collectives between stages is done here with sums over the
    devices' partial results (hap_add): the All-Reduce of the Wo / W2 products in the forward and
    of the bwd-data products in the backward ("tensor" style).  In "data" style a device's rows
    never meet another device's, so no sums are needed (weight gradients stay per-device partials).
    """

    def __init__(self, style, B, S, hidden, heads, d, ffn, head_offsets, ffn_offsets, batch_offsets, params, x, dy):
        self.style, self.hidden, self.S = style, hidden, S
        self.params, self.x, self.dy = params, x, dy
        m = (len(head_offsets) if style == "tensor" else len(batch_offsets)) - 1
        self.shards = [EncoderShard(style, j, B, S, hidden, heads, d, ffn, head_offsets, ffn_offsets, batch_offsets, params) for j in range(m)]
        N = B * S
        self.N = N
        z = lambda: torch.zeros((N, hidden), dtype=x.dtype, device=x.device)
        self.x1, self.y, self.dx1, self.dx, self.red = z(), z(), z(), z(), z()
        self.db2 = torch.zeros((hidden,), dtype=torch.float32, device=x.device)
        self.dbo = torch.zeros((hidden,), dtype=torch.float32, device=x.device)
        self.ws = torch.empty((max(hap.hap_colsum_workspace(N, hidden), 256),), dtype=torch.uint8, device=x.device)

    def _add(self, n, a, b, bias, out):
        hap.hap_add(n, self.hidden, hap.BF16, a, self.hidden, b, self.hidden, bias, out, self.hidden)

    def _reduce(self, parts, out):
        """out = sum of the devices' partial tensors (the All-Reduce)."""
        if len(parts) == 1:
            out.copy_(parts[0]); return
        self._add(self.N, parts[0], parts[1], None, out)
        for p in parts[2:]:
            self._add(self.N, out, p, None, out)

    def forward(self):
        p, N = self.params, self.N
        if self.style == "tensor":
            for s in self.shards:
                s.attn_forward(self.x)
            self._reduce([s.attn_part for s in self.shards], self.red)
            self._add(N, self.x, self.red, p["bo"], self.x1)
            for s in self.shards:
                s.mlp_forward(self.x1)
            self._reduce([s.mlp_part for s in self.shards], self.red)
            self._add(N, self.x1, self.red, p["b2"], self.y)
        else:
            for s in self.shards:      # a device with an empty batch shard runs the same calls on zero rows
                xr, x1r, yr = s.rows(self.x), s.rows(self.x1), s.rows(self.y)
                s.attn_forward(xr)
                self._add(s.N, xr, s.attn_part, p["bo"], x1r)
                s.mlp_forward(x1r)
                self._add(s.N, x1r, s.mlp_part, p["b2"], yr)

    def backward(self):
        N = self.N
        if self.style == "tensor":
            s0 = self.shards[0]
            for s in self.shards:
                s.mlp_backward(self.dy)
            self._reduce([s.dln2_part for s in self.shards], self.red)
            s0.ln2_backward(self.x1, self.red, self.dy, self.dx1)    # replicated: every device computes the same
            for s in self.shards:
                s.attn_backward(self.dx1)
            self._reduce([s.dln1_part for s in self.shards], self.red)
            s0.ln1_backward(self.x, self.red, self.dx1, self.dx)
        else:
            for s in self.shards:      # an empty shard's weight-gradient partials come out as zeros (empty sums)
                xr, x1r, dyr, dx1r, dxr = (s.rows(t) for t in (self.x, self.x1, self.dy, self.dx1, self.dx))
                s.mlp_backward(dyr)
                s.ln2_backward(x1r, s.dln2_part, dyr, dx1r)
                s.attn_backward(dx1r)
                s.ln1_backward(xr, s.dln1_part, dx1r, dxr)
        hap.hap_colsum(N, self.hidden, hap.BF16, self.dy, self.hidden, self.db2, self.ws)
        hap.hap_colsum(N, self.hidden, hap.BF16, self.dx1, self.hidden, self.dbo, self.ws)
