"""Single-device reference of the layers the workloads are built from.

The correctness criterion of the paper (Sec. 4.1) is that the distributed
program yields what the single-device graph yields, so the oracle for any
sharded execution is the unsharded layer evaluated once in float64, with every
intermediate kept so that tests can slice (batch / feature shards) or sum
(reduction partials) and compare.

  mlp_block:      H = gelu(X W1 + b1);  Out = H W2 + b2
  encoder_layer:  pre-LayerNorm Transformer encoder layer
                  x1 = x + Attn(LN1(x)) Wo + bo;  y = x1 + MLP(LN2(x1))
"""
from __future__ import annotations

import numpy as np

from . import attention, pointwise


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def mlp_block(X, W1, b1, W2, b2, dOut):
    X, W1, b1, W2, b2, dOut = map(_f64, (X, W1, b1, W2, b2, dOut))
    pre = X @ W1 + b1
    H = pointwise.gelu(pre)
    out = H @ W2 + b2
    dH = dOut @ W2.T
    dW2 = H.T @ dOut
    db2 = dOut.sum(axis=0)
    dP = dH * pointwise.gelu_grad(pre)
    dX = dP @ W1.T
    dW1 = X.T @ dP
    db1 = dP.sum(axis=0)
    return dict(pre=pre, H=H, out=out, dH=dH, dP=dP, dX=dX, dW1=dW1, db1=db1, dW2=dW2, db2=db2)



def moe_ffn_block(X, W1, b1, W2, b2, dOut, rows=None):
    """Expert feed-forward layer of an MoE block (Sec. 7.6): per expert e, on its rows[e] tokens,
    H_e = gelu(X_e W1_e + b1_e), Out_e = H_e W2_e + b2_e, and the gradients of L = sum(Out * dOut).
    X, dOut [E x C x hidden]; W1 [E x hidden x ffn]; W2 [E x ffn x hidden]; biases [E x ffn], [E x hidden]."""
    from . import moe
    H, pre = moe.moe_linear_fwd(X, W1, b1, rows, act=True)
    out, _ = moe.moe_linear_fwd(H, W2, b2, rows, act=False)
    dH, dW2, db2 = moe.moe_linear_bwd(H, W2, None, dOut, rows, act=False)
    dX, dW1, db1 = moe.moe_linear_bwd(X, W1, pre, dH, rows, act=True)
    return dict(pre=pre, H=H, out=out, dH=dH, dX=dX, dW1=dW1, db1=db1, dW2=dW2, db2=db2)

def _split_heads(t, batch, seq, heads, d):
    return t.reshape(batch, seq, heads, d).transpose(0, 2, 1, 3)


def _merge_heads(t):
    b, h, s, d = t.shape
    return t.transpose(0, 2, 1, 3).reshape(b * s, h * d)


def encoder_layer(x, p, dY, batch, seq, heads, head_dim):
    """x, dY: [batch*seq, hidden].  p: dict of g1,be1,Wq,bq,Wk,bk,Wv,bv,Wo,bo,g2,be2,W1,b1,W2,b2.

    Returns every forward intermediate and every gradient of L = sum(y * dY).
    """
    x, dY = _f64(x), _f64(dY)
    p = {k: _f64(v) for k, v in p.items()}
    r = {}
    ln1, _, _ = pointwise.layernorm_fwd(x, p["g1"], p["be1"])
    q = ln1 @ p["Wq"] + p["bq"]
    k = ln1 @ p["Wk"] + p["bk"]
    v = ln1 @ p["Wv"] + p["bv"]
    qh, kh, vh = (_split_heads(t, batch, seq, heads, head_dim) for t in (q, k, v))
    oh, lse = attention.attn_fwd(qh, kh, vh)
    o = _merge_heads(oh)
    attn_out = o @ p["Wo"] + p["bo"]
    x1 = x + attn_out
    ln2, _, _ = pointwise.layernorm_fwd(x1, p["g2"], p["be2"])
    pre = ln2 @ p["W1"] + p["b1"]
    H = pointwise.gelu(pre)
    mlp_out = H @ p["W2"] + p["b2"]
    y = x1 + mlp_out
    r.update(ln1=ln1, q=q, k=k, v=v, o=o, lse=lse, attn_out=attn_out, x1=x1, ln2=ln2, pre=pre, H=H,
             mlp_out=mlp_out, y=y)
    # backward
    dH = dY @ p["W2"].T
    r["dW2"] = H.T @ dY
    r["db2"] = dY.sum(axis=0)
    dP = dH * pointwise.gelu_grad(pre)
    r["dW1"] = ln2.T @ dP
    r["db1"] = dP.sum(axis=0)
    dln2 = dP @ p["W1"].T
    dx1_ln, r["dg2"], r["dbe2"] = pointwise.layernorm_bwd(x1, p["g2"], dln2)
    dx1 = dY + dx1_ln
    r["dWo"] = o.T @ dx1
    r["dbo"] = dx1.sum(axis=0)
    do = dx1 @ p["Wo"].T
    doh = _split_heads(do, batch, seq, heads, head_dim)
    dqh, dkh, dvh = attention.attn_bwd(qh, kh, vh, doh)
    dq, dk, dv = _merge_heads(dqh), _merge_heads(dkh), _merge_heads(dvh)
    r["dWq"], r["dWk"], r["dWv"] = ln1.T @ dq, ln1.T @ dk, ln1.T @ dv
    r["dbq"], r["dbk"], r["dbv"] = dq.sum(axis=0), dk.sum(axis=0), dv.sum(axis=0)
    dln1 = dq @ p["Wq"].T + dk @ p["Wk"].T + dv @ p["Wv"].T
    dx_ln, r["dg1"], r["dbe1"] = pointwise.layernorm_bwd(x, p["g1"], dln1)
    r["dx"] = dx1 + dx_ln
    r.update(dH=dH, dP=dP, dln2=dln2, dx1=dx1, do=do, dq=dq, dk=dk, dv=dv, dln1=dln1)
    return r
