"""GPU parity of configs 4 and 5 at their stated sizes, in the launch configuration bench.py times: the whole
layer of every virtual device (batch 16 x 1024 tokens, hidden 2048; batch 256 x 197 tokens, hidden 1024), the
ffn-sharded MLP of config 5 over all 50432 tokens, and the sufficient-factor rebuild of both MLP weight
gradients with a contraction of 50432 rows in five ragged segments.  The float64 single-device oracle runs on
the full tensors (a few TFLOP of BLAS-backed numpy: seconds on the GPU machine's cores) and every element of every
output tensor is compared."""
import numpy as np
import pytest

import hapgen
from hapgen import TensorId as T
from oracle import layers as olay, sfb as osfb

pytestmark = pytest.mark.gpu

from gpu_util import gen, empty, host, check, relerr  # noqa: E402
from test_gpu_layers import _check_layer, ratios_offsets  # noqa: E402


@pytest.fixture(scope="module")
def hap():
    import paper_2401_05965_amd as h
    return h


def test_cfg4_encoder_layer_full_size(hap):
    """Config 4 as stated: batch 16 x seq 1024, hidden 2048, heads (5, 5, 3, 3) of 16 x 128, ffn (2731, 2731, 1365, 1365) of
    8192: all four devices' shards (the 16384-token launches), their partial products summed as the All-Reduce would."""
    w = hapgen.WORKLOADS["cfg4_encoder_bf16"]; d = w.dims
    sizes, _ = ratios_offsets(hap, w.speeds, d["heads"])
    assert sizes == [5, 5, 3, 3]
    sizes, _ = ratios_offsets(hap, w.speeds, d["ffn"])
    assert sizes == [2731, 2731, 1365, 1365]
    _check_layer(hap, "tensor", B=d["batch"], S=d["seq"], hidden=d["hidden"], heads=d["heads"], d=d["head_dim"], ffn=d["ffn"], speeds=w.speeds)


def test_cfg5_vit_layer_full_size(hap):
    """Config 5's batch-sharded layer as stated: 256 samples x 197 tokens over five devices -> (79, 63, 63, 31, 20) samples,
    hidden 1024, 16 heads x 64, ffn 4096; device 0's 15563-token and device 4's 3940-token launches included."""
    w = hapgen.WORKLOADS["cfg5_vit_bf16"]; d = w.dims
    sizes, _ = ratios_offsets(hap, w.speeds, d["batch"])
    assert sizes == [79, 63, 63, 31, 20]
    _check_layer(hap, "data", B=d["batch"], S=d["seq"], hidden=d["hidden"], heads=d["heads"], d=d["head_dim"], ffn=d["ffn"], speeds=w.speeds)


def test_cfg5_mlp_ffn_sharded_full_size(hap):
    """Config 5's MLP with the ffn axis sharded (1261, 1008, 1008, 504, 315 of 4096) over all 50432 tokens: every device's
    slices against the unsharded block, the partial outputs and input gradients summed over the devices."""
    from paper_2401_05965_amd.programs import MlpShard
    w = hapgen.WORKLOADS["cfg5_vit_bf16"]; d = w.dims
    tokens, hidden, ffn = d["batch"] * d["seq"], d["hidden"], d["ffn"]
    sizes, offs = ratios_offsets(hap, w.speeds, ffn)
    assert sizes == [1261, 1008, 1008, 504, 315]
    Xh, Xd = gen(5, T.X, (tokens, hidden), 1.0, "bf16"); W1h, W1d = gen(5, T.W, (hidden, ffn), 0.02, "bf16")
    b1h, b1d = gen(5, T.BIAS, (ffn,), 0.02, "bf16"); W2h, W2d = gen(5, T.W2, (ffn, hidden), 0.02, "bf16")
    dOh, dOd = gen(5, T.DY, (tokens, hidden), 1.0, "bf16")
    ref = olay.mlp_block(Xh, W1h, b1h, W2h, np.zeros(hidden), dOh)
    out = np.zeros((tokens, hidden)); dX = np.zeros((tokens, hidden))
    for j in range(len(sizes)):
        s = MlpShard(tokens, hidden, ffn, offs, j, Xd, W1d, b1d, W2d, dOd)
        s.forward(); s.backward()
        c = slice(offs[j], offs[j + 1]); f = s.f
        for n, got, want in (("H", host(s.H)[:, :f], ref["H"][:, c]), (s.dH_holds, host(s.dH)[:, :f], ref[s.dH_holds][:, c]),
                             ("dW1", host(s.dW1)[:, :f], ref["dW1"][:, c]), ("db1", host(s.db1)[:f], ref["db1"][c]),
                             ("dW2", host(s.dW2)[:f], ref["dW2"][c])):
            e = check(f"{n}_{j}", got, want, "bf16")
            print(f"cfg5 mlp device {j} (ffn {f}) {n}: {e:.3e}")
        out += host(s.P); dX += host(s.dX)
        del s
    e_out, e_dx = relerr(out, ref["out"]), relerr(dX, ref["dX"])
    print(f"cfg5 mlp summed partials: out {e_out:.3e}, dX {e_dx:.3e}")
    assert e_out <= 2e-2 and e_dx <= 2e-2


@pytest.mark.parametrize("with_workspace", [True, False])
def test_cfg5_sfb_rebuild_full_size(hap, with_workspace):
    """Config 5's second MLP program: dW1 [1024 x 4096] and dW2 [4096 x 1024] rebuilt from five devices' gathered factors,
    token counts 197 x (79, 63, 63, 31, 20) = 50432 contracted rows; with the optional scratch (the contraction is split
    over idle compute units, across the ragged segment boundaries) and without it."""
    w = hapgen.WORKLOADS["cfg5_vit_bf16"]; d = w.dims
    sizes, boffs = ratios_offsets(hap, w.speeds, d["batch"])
    rows = [d["seq"] * b for b in sizes]
    assert sum(rows) == 50432
    hidden, ffn = d["hidden"], d["ffn"]
    Xh, Xd, Yh, Yd = [], [], [], []
    for i, r in enumerate(rows):
        a, b = gen(5, T.SFB_X + i, (r, hidden), 1.0, "bf16"); Xh.append(a); Xd.append(b)
        a, b = gen(5, T.SFB_DY + i, (r, ffn), 1.0, "bf16"); Yh.append(a); Yd.append(b)
    ws = empty((max(hap.hap_sfb_workspace(len(rows), rows, hidden, ffn), 16),), "u8") if with_workspace else None
    dW1 = empty((hidden, ffn), "f32", float("nan"))
    hap.hap_sfb_grad(Xd, Yd, rows, hidden, ffn, hidden, ffn, hap.BF16, dW1, ffn, ws=ws)
    e1 = check("cfg5 sfb dW1", host(dW1), osfb.sfb_grad(Xh, Yh, rows), "bf16")
    dW2 = empty((ffn, hidden), "f32", float("nan"))
    hap.hap_sfb_grad(Yd, Xd, rows, ffn, hidden, ffn, hidden, hap.BF16, dW2, hidden, ws=ws)
    e2 = check("cfg5 sfb dW2", host(dW2), osfb.sfb_grad(Yh, Xh, rows), "bf16")
    print(f"cfg5 sfb (workspace {with_workspace}): dW1 {e1:.3e}, dW2 {e2:.3e}")
