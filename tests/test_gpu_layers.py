"""GPU parity of whole sharded layers against the single-device oracle (Sec. 4.1: the distributed
program must produce what the single-device graph produces).  Reduced sizes that still span
several tiles, ragged shard widths and uneven head / batch counts."""
import numpy as np
import pytest

import hapgen
from hapgen import TensorId as T
from oracle import layers as olay, lp as olp, rounding as ornd, sfb as osfb

pytestmark = pytest.mark.gpu

from gpu_util import gen, empty, host, check, relerr, torch_mod  # noqa: E402


@pytest.fixture(scope="module")
def hap():
    import paper_2401_05965_amd as h
    return h


def make_params(seed, hidden, ffn, sw):
    names = [("Wq", T.WQ, (hidden, hidden), sw), ("Wk", T.WK, (hidden, hidden), sw), ("Wv", T.WV, (hidden, hidden), sw),
             ("Wo", T.WO, (hidden, hidden), sw), ("W1", T.W, (hidden, ffn), sw), ("W2", T.W2, (ffn, hidden), sw)]
    small = [("bq", hidden), ("bk", hidden), ("bv", hidden), ("bo", hidden), ("b1", ffn), ("b2", hidden), ("be1", hidden), ("be2", hidden)]
    ph, pd = {}, {}
    for n, t, shp, s in names:
        ph[n], pd[n] = gen(seed, t, shp, s, "bf16")
    for i, (n, sz) in enumerate(small):
        ph[n], pd[n] = gen(seed, T.MISC + i, (sz,), 0.1, "bf16")
    for i, n in enumerate(("g1", "g2")):
        h_, d_ = gen(seed, T.MISC + 20 + i, (hidden,), 0.1, "bf16")
        # gamma = 1 + small, snapped to bf16 so host and device agree exactly
        bits = hapgen.to_bf16_bits((1.0 + h_).astype(np.float32))
        ph[n] = hapgen.from_bf16_bits(bits).astype(np.float64)
        torch = torch_mod()
        pd[n] = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()
    return ph, pd


def ratios_offsets(hap, speeds, n, granule=1):
    r, _ = hap.hap_shard_ratios(speeds, [(1.0, 0, 0, 0)])
    sizes, offs = hap.hap_round_shards(r, n, granule)
    assert (sizes, offs) == ornd.round_shards(olp.shard_ratios(speeds, [(1.0, 0, 0, 0)])[0], n, granule)   # bit-exact ranges
    return sizes, offs


@pytest.mark.parametrize("fuse_act_bwd", [True, False])
def test_mlp_block_ffn_sharded_three_devices(hap, fuse_act_bwd):
    """cfg2 at reduced size: ffn sharded by speeds (1, 0.6, 0.35); partial outputs summed = unsharded block.  With the GeLU
    backward folded into fc2's bwd-data epilogue (the buffer dH then holds dP = dH * gelu'(pre)) and as a pass of its own."""
    from paper_2401_05965_amd.programs import MlpShard
    tokens, hidden, ffn = 640, 384, 1111
    sizes, offs = ratios_offsets(hap, (1.0, 0.6, 0.35), ffn)
    Xh, Xd = gen(0, T.X, (tokens, hidden), 1.0, "bf16"); W1h, W1d = gen(0, T.W, (hidden, ffn), 0.05, "bf16")
    b1h, b1d = gen(0, T.BIAS, (ffn,), 0.1, "bf16"); W2h, W2d = gen(0, T.W2, (ffn, hidden), 0.05, "bf16")
    dOh, dOd = gen(0, T.DY, (tokens, hidden), 1.0, "bf16")
    ref = olay.mlp_block(Xh, W1h, b1h, W2h, np.zeros(hidden), dOh)
    out = np.zeros((tokens, hidden)); dX = np.zeros((tokens, hidden))
    for j in range(3):
        s = MlpShard(tokens, hidden, ffn, offs, j, Xd, W1d, b1d, W2d, dOd, fuse_act_bwd=fuse_act_bwd)
        s.forward(); s.backward()
        c = slice(offs[j], offs[j + 1]); f = s.f
        check(f"H_{j}", host(s.H)[:, :f], ref["H"][:, c], "bf16")
        check(f"{s.dH_holds}_{j}", host(s.dH)[:, :f], ref[s.dH_holds][:, c], "bf16")
        check(f"dW1_{j}", host(s.dW1)[:, :f], ref["dW1"][:, c], "bf16")
        check(f"db1_{j}", host(s.db1)[:f], ref["db1"][c], "bf16")
        check(f"dW2_{j}", host(s.dW2)[:f], ref["dW2"][c], "bf16")
        out += host(s.P); dX += host(s.dX)
    assert relerr(out, ref["out"]) <= 2e-2 and relerr(dX, ref["dX"]) <= 2e-2


def _check_layer(hap, style, B, S, hidden, heads, d, ffn, speeds):
    from paper_2401_05965_amd.programs import EncoderLayerProgram
    ph, pd = make_params(1, hidden, ffn, 0.05 if hidden < 1024 else 0.02)
    xh, xd = gen(1, T.X, (B * S, hidden), 1.0, "bf16"); dyh, dyd = gen(1, T.DY, (B * S, hidden), 1.0, "bf16")
    _, hoffs = ratios_offsets(hap, speeds, heads)
    _, foffs = ratios_offsets(hap, speeds, ffn)
    _, boffs = ratios_offsets(hap, speeds, B)
    prog = EncoderLayerProgram(style, B, S, hidden, heads, d, ffn, hoffs, foffs, boffs, pd, xd, dyd)
    for s in prog.shards:
        if s.N == 0:      # an empty batch shard: its partial gradients must be WRITTEN as zeros, not left as they were
            for t in (s.dWqkv, s.dWo, s.dW1, s.dW2, s.dbqkv, s.db1, s.dg1, s.dbe1, s.dg2, s.dbe2):
                t.fill_(float("nan"))
    prog.forward(); prog.backward()
    ref = olay.encoder_layer(xh, ph, dyh, B, S, heads, d)
    for n, t in (("x1", prog.x1), ("y", prog.y), ("dx1", prog.dx1), ("dx", prog.dx), ("db2", prog.db2), ("dbo", prog.dbo)):
        check(f"{style} {n}", host(t), ref[n], "bf16")
    acc = {}
    for j, s in enumerate(prog.shards):
        hd, f = s.hd, s.f
        if style == "tensor":
            c = slice(hoffs[j] * d, hoffs[j + 1] * d); fc = slice(foffs[j], foffs[j + 1])
            if hd:
                got = host(s.dWqkv)
                for i, n in enumerate(("dWq", "dWk", "dWv")):
                    check(f"{n}_{j}", got[:, i * hd:(i + 1) * hd], ref[n][:, c], "bf16")
                gb = host(s.dbqkv)
                for i, n in enumerate(("dbq", "dbk", "dbv")):
                    if n == "dbk":
                        # exactly zero in exact arithmetic (a shift of every key leaves softmax unchanged): the
                        # device's value is the rounding residue of a cancelling sum, bounded by eps_bf16 * sum|dk|
                        assert np.abs(gb[i * hd:(i + 1) * hd]).max() <= 2.0 ** -8 * np.abs(ref["dk"][:, c]).sum(0).max()
                        continue
                    check(f"{n}_{j}", gb[i * hd:(i + 1) * hd], ref[n][c], "bf16")
                check(f"dWo_{j}", host(s.dWo)[:hd], ref["dWo"][c], "bf16")
                check(f"o_{j}", host(s.o)[:, :hd], ref["o"][:, c], "bf16")
            if f:
                check(f"dW1_{j}", host(s.dW1)[:, :f], ref["dW1"][:, fc], "bf16")
                check(f"db1_{j}", host(s.db1)[:f], ref["db1"][fc], "bf16")
                check(f"dW2_{j}", host(s.dW2)[:f], ref["dW2"][fc], "bf16")
        else:
            H = hidden
            got = host(s.dWqkv)
            parts = {"dWq": got[:, :H], "dWk": got[:, H:2 * H], "dWv": got[:, 2 * H:3 * H], "dWo": host(s.dWo), "dW1": host(s.dW1)[:, :ffn],
                     "dW2": host(s.dW2), "db1": host(s.db1), "dg1": host(s.dg1), "dbe1": host(s.dbe1), "dg2": host(s.dg2), "dbe2": host(s.dbe2)}
            gb = host(s.dbqkv)
            parts.update(dbq=gb[:H], dbk=gb[H:2 * H], dbv=gb[2 * H:])
            for n, v in parts.items():
                acc[n] = acc.get(n, 0) + v
    if style == "tensor":
        s0 = prog.shards[0]
        for n, t in (("dg1", s0.dg1), ("dbe1", s0.dbe1), ("dg2", s0.dg2), ("dbe2", s0.dbe2)):
            check(f"tensor {n}", host(t), ref[n], "bf16")
    else:
        # per-device weight gradients are partial sums over the batch: their sum is the all-reduced gradient
        for n, v in acc.items():
            if n == "dbk":
                assert np.abs(v).max() <= 2.0 ** -8 * np.abs(ref["dk"]).sum(0).max()
                continue
            assert relerr(v, ref[n]) <= 2e-2, (n, relerr(v, ref[n]))


def test_encoder_layer_heads_and_ffn_sharded(hap):
    """cfg4 at reduced size: 4 devices with speeds (1,1,.5,.5): uneven head counts, ragged ffn widths."""
    _check_layer(hap, "tensor", B=2, S=200, hidden=768, heads=6, d=128, ffn=1000, speeds=(1.0, 1.0, 0.5, 0.5))


def test_vit_layer_batch_sharded(hap):
    """cfg5 at reduced size: 5 devices with speeds (1,.8,.8,.4,.25): batch slices, seq 197, head_dim 64."""
    _check_layer(hap, "data", B=13, S=197, hidden=256, heads=4, d=64, ffn=520, speeds=(1.0, 0.8, 0.8, 0.4, 0.25))


def test_vit_layer_batch_sharded_with_an_empty_device(hap):
    """Four samples over five devices (1, .8, .8, .4, .25) round to (1, 1, 1, 1, 0): the last device owns no rows, runs the
    same calls on zero rows and contributes all-zero partial weight gradients (its buffers are NaN-filled beforehand)."""
    sizes, _ = ratios_offsets(hap, (1.0, 0.8, 0.8, 0.4, 0.25), 4)
    assert sizes == [1, 1, 1, 1, 0]
    _check_layer(hap, "data", B=4, S=197, hidden=256, heads=4, d=64, ffn=520, speeds=(1.0, 0.8, 0.8, 0.4, 0.25))


def test_vit_mlp_sfb_weight_gradients(hap):
    """cfg5's second program for the MLP: batch-sharded devices all-gather their factors and each rebuilds
    dW1 = LN2^T dP and dW2 = H^T dOut over the whole batch (uneven token counts 197*b_j)."""
    torch = torch_mod()
    B, S, hidden, ffn = 13, 197, 256, 520
    _, boffs = ratios_offsets(hap, (1.0, 0.8, 0.8, 0.4, 0.25), B)
    rows = [S * (boffs[j + 1] - boffs[j]) for j in range(5)]
    Xh, Xd = gen(2, T.X, (B * S, hidden), 1.0, "bf16"); dPh, dPd = gen(2, T.DY, (B * S, ffn), 1.0, "bf16")
    toks = [S * b for b in boffs]
    Xs = [Xd[toks[j]:toks[j + 1]] for j in range(5)]; dPs = [dPd[toks[j]:toks[j + 1]] for j in range(5)]
    dW1 = empty((hidden, ffn), "f32", float("nan"))
    hap.hap_sfb_grad(Xs, dPs, rows, hidden, ffn, hidden, ffn, hap.BF16, dW1, ffn)
    check("sfb dW1", host(dW1), Xh.T @ dPh, "bf16")
    check("sfb dW1 vs factor sum", host(dW1), osfb.sfb_grad([Xh[toks[j]:toks[j + 1]] for j in range(5)], [dPh[toks[j]:toks[j + 1]] for j in range(5)], rows), "bf16")
    dW2 = empty((ffn, hidden), "f32", float("nan"))
    hap.hap_sfb_grad(dPs, Xs, rows, ffn, hidden, ffn, hidden, hap.BF16, dW2, hidden)
    check("sfb dW2", host(dW2), dPh.T @ Xh, "bf16")


def test_cfg4_encoder_layer_full_widths(hap):
    """cfg4 with its real widths (hidden 2048, 16 heads x 128 -> 5,5,3,3 heads, ffn 8192 -> 2731,2731,1365,1365, seq 1024)
    and a reduced batch (2 of 16) so the float64 single-device oracle finishes in seconds."""
    w = hapgen.WORKLOADS["cfg4_encoder_bf16"]; d = w.dims
    _check_layer(hap, "tensor", B=2, S=d["seq"], hidden=d["hidden"], heads=d["heads"], d=d["head_dim"], ffn=d["ffn"], speeds=w.speeds)


def test_cfg5_vit_layer_full_widths(hap):
    """cfg5 with its real widths (hidden 1024, 16 heads x 64, 197 tokens, ffn 4096) and batch 26 of 256
    (5 devices -> 8,6,6,3,3 samples)."""
    w = hapgen.WORKLOADS["cfg5_vit_bf16"]; d = w.dims
    _check_layer(hap, "data", B=26, S=d["seq"], hidden=d["hidden"], heads=d["heads"], d=d["head_dim"], ffn=d["ffn"], speeds=w.speeds)


def test_encoder_layer_replays_from_a_hip_graph(hap):
    """A whole bf16 encoder layer of all four devices' shards (projections, attention, LayerNorm, GeLU, residuals, every
    gradient: about 150 kernels incl. split-K reductions) captured once and replayed: the library only launches kernels on
    the caller's stream, so every replay - with eager work and synchronisations in between - is bit-identical to eager."""
    from paper_2401_05965_amd.programs import EncoderLayerProgram
    torch = torch_mod()
    B, S, hidden, heads, d, ffn, speeds = 2, 200, 768, 6, 128, 1000, (1.0, 1.0, 0.5, 0.5)
    _, pd = make_params(1, hidden, ffn, 0.05)
    _, xd = gen(1, T.X, (B * S, hidden), 1.0, "bf16"); _, dyd = gen(1, T.DY, (B * S, hidden), 1.0, "bf16")
    _, hoffs = ratios_offsets(hap, speeds, heads)
    _, foffs = ratios_offsets(hap, speeds, ffn)
    _, boffs = ratios_offsets(hap, speeds, B)
    prog = EncoderLayerProgram("tensor", B, S, hidden, heads, d, ffn, hoffs, foffs, boffs, pd, xd, dyd)

    def step():
        prog.forward(); prog.backward()
    outs = {"x1": prog.x1, "y": prog.y, "dx1": prog.dx1, "dx": prog.dx, "db2": prog.db2, "dbo": prog.dbo}
    for j, s in enumerate(prog.shards):
        # the valid parts of the compact buffers (the library never writes their padding)
        outs.update({f"dWqkv{j}": s.dWqkv[:, :3 * s.hd], f"dWo{j}": s.dWo[:s.hd], f"dW1{j}": s.dW1[:, :s.f], f"dW2{j}": s.dW2[:s.f], f"db1{j}": s.db1[:s.f]})
    step()
    torch.cuda.synchronize()
    want = {k: v.clone() for k, v in outs.items()}
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        step()
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for rep in range(3):
        for v in outs.values():
            v.fill_(float(rep + 1))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in outs:
            assert torch.equal(outs[k], want[k]), (rep, k)
        step()
        torch.cuda.synchronize()
