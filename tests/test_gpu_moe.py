"""GPU parity of the expert-sharded MoE layer (Sec. 7.6, uneven placement of experts) against the CPU
oracle, through the C ABI.  Tolerances as for the linear layers: max|err| / max|ref| per tensor
<= 2e-2 (bf16 in, fp32 accumulate) or 1e-5 (fp32); expert ranges come from the LP + rounding and are
compared bit-exactly.  Buffer rows without a token are poisoned with NaN on input and must come back
untouched on output.
"""
import numpy as np
import pytest

from hapgen import TensorId as T
from oracle import moe as omoe, lp as olp, rounding as ornd

pytestmark = pytest.mark.gpu

from gpu_util import gen, empty, host, check, torch_mod  # noqa: E402

DT = {"bf16": 1, "f32": 0}
SENTINEL = 768.0            # pre-filled into outputs: rows the library must leave untouched keep it


@pytest.fixture(scope="module")
def hap():
    import paper_2401_05965_amd as h
    return h


def expert_offsets(hap, speeds, experts):
    r, _ = hap.hap_shard_ratios(speeds, [(1.0, 0, 0, 0)])
    sizes, offs = hap.hap_round_shards(r, experts, 1)
    assert (sizes, offs) == ornd.round_shards(olp.shard_ratios(speeds, [(1.0, 0, 0, 0)])[0], experts, 1)
    return sizes, offs


def run_moe_case(hap, dtype, E, C, in_f, out_f, offs, rows, act, bias, full, dw_dtype=None, pad=0, seed=9, fwd_ws=False):
    torch = torch_mod()
    dw_dtype = dw_dtype or dtype
    ldx, ldw, ldy = in_f + pad, out_f + pad, out_f + pad
    Xh, _ = gen(seed, T.X, (E, C, in_f), 1.0, dtype); Wh, _ = gen(seed, T.W, (E, in_f, out_f), 0.05, dtype)
    bh, _ = gen(seed, T.BIAS, (E, out_f), 0.5, dtype) if bias else (None, None)
    dYh, _ = gen(seed, T.DY, (E, C, out_f), 1.0, dtype)
    nrows = np.full(E, C) if rows is None else np.asarray(rows)
    live = np.arange(C)[None, :] < nrows[:, None]                       # [E, C]

    def padded(vals, ld, poison_rows):
        """[E, R, cols] host values -> device buffer [E, R, ld]; pad columns and (optionally) token-less rows are NaN."""
        buf = np.full(vals.shape[:2] + (ld,), np.nan)
        buf[:, :, :vals.shape[2]] = vals
        if poison_rows:
            buf[~live] = np.nan
        t = torch.from_numpy(buf.astype(np.float32)).cuda()
        return t.to(torch.bfloat16) if dtype == "bf16" else t
    Xd, dYd = padded(Xh, ldx, True), padded(dYh, ldy, True)
    Wd = padded(Wh, ldw, False)
    bd = (torch.from_numpy(bh.astype(np.float32)).cuda().to(torch.bfloat16 if dtype == "bf16" else torch.float32)) if bias else None
    rows_d = torch.from_numpy(nrows.astype(np.int32)).cuda() if rows is not None else None

    Yo, preo = omoe.moe_linear_fwd(Xh, Wh, bh, rows, act)
    dXo, dWo, dbo = omoe.moe_linear_bwd(Xh, Wh, preo, dYh, rows, act)
    m = len(offs) - 1
    worst = 0.0
    for j in range(m):
        lo, hi = offs[j], offs[j + 1]
        n = hi - lo
        s = slice(lo, hi)
        if full:
            desc = hap.MoeDesc(E, C, in_f, out_f, offs, DT[dtype], act=int(act), has_bias=bias, ldx=ldx, ldw=ldw, ldy=ldy, operands_are_full=True)
            Xj, Wj, bj, dYj, rj = Xd, Wd, bd, dYd, rows_d
            ne, base = E, lo
        else:
            desc = hap.MoeDesc(E, C, in_f, out_f, offs, DT[dtype], act=int(act), has_bias=bias, ldx=ldx, ldw=ldw, ldy=ldy, operands_are_full=False)
            Xj, Wj, dYj = Xd[s].contiguous(), Wd[s].contiguous(), dYd[s].contiguous()
            bj = bd[s].contiguous() if bias else None
            rj = rows_d[s].contiguous() if rows is not None else None
            ne, base = n, 0
            if n == 0:
                Xj = Wj = dYj = bj = rj = None
        Y = empty((ne, C, ldy), dtype, SENTINEL); P = empty((ne, C, ldy), dtype, SENTINEL) if act else None
        dX = empty((ne, C, ldx), dtype, SENTINEL); dW = empty((ne, in_f, ldw), dw_dtype, SENTINEL); db = empty((ne, out_f), "f32", SENTINEL)
        ws = empty((max(hap.hap_moe_linear_bwd_workspace(desc, j), hap.hap_moe_linear_fwd_workspace(desc, j), 16),), "u8")
        hap.hap_moe_linear_fwd(desc, j, Xj, Wj, bj if bias else None, rj, Y, P, ws if fwd_ws else None)
        hap.hap_moe_linear_bwd(desc, j, Xj, Wj, P, dYj, rj, dX, dW, DT[dw_dtype], db, ws)
        got = {k: host(v) for k, v in (("Y", Y), ("dX", dX), ("dW", dW), ("db", db))}
        if act:
            got["P"] = host(P)
        own = slice(base, base + n)
        lv = live[s]
        for name, ref, width in (("Y", Yo, out_f), ("P", preo, out_f), ("dX", dXo, in_f)):
            if name not in got:
                continue
            g = got[name][own][:, :, :width]
            if n and lv.any():
                worst = max(worst, check(f"{name} dev{j}", g[lv], ref[s][lv], dtype))
            assert (g[~lv] == SENTINEL).all(), f"{name}: rows without a token were written"
            assert (got[name][own][:, :, width:] == SENTINEL).all(), f"{name}: pad columns were written"
        if n:
            worst = max(worst, check(f"dW dev{j}", got["dW"][own][:, :, :out_f], dWo[s], dtype))
            assert (got["dW"][own][:, :, out_f:] == SENTINEL).all(), "dW: pad columns were written"
            worst = max(worst, check(f"db dev{j}", got["db"][own], dbo[s], dtype))
        if full:   # the other devices' experts are not touched
            other = np.ones(E, bool); other[s] = False
            for name in got:
                assert (got[name][other] == SENTINEL).all(), f"{name}: experts of another device were written"
    return worst


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("full", [True, False])
def test_moe_uneven_experts_ragged_rows(hap, dtype, full):
    """7 experts over 5 devices with unequal speeds -> (3, 2, 1, 1, 0) experts; token counts ragged incl. 0 and full;
    several 128- and 256-tiles per expert with ragged tails in every dimension."""
    sizes, offs = expert_offsets(hap, (1.0, 1.0, 0.5, 0.5, 0.01), 7)
    assert sizes == [3, 2, 1, 1, 0]
    rows = [300, 77, 0, 300, 1, 256, 129]
    run_moe_case(hap, dtype, 7, 300, 200, 328, offs, rows, act=True, bias=True, full=full)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_moe_all_rows_valid_no_activation(hap, dtype):
    """rows = NULL (capacity-padded dispatch: every buffer row counts), no bias, no activation, fp32 dW from bf16."""
    sizes, offs = expert_offsets(hap, (1.0, 0.6), 5)
    assert sizes == [3, 2]
    run_moe_case(hap, dtype, 5, 160, 136, 264, offs, None, act=False, bias=False, full=True, dw_dtype="f32")


def test_moe_big_tiles_bf16(hap):
    """Enough experts x tiles that the 256x256 kernel is chosen; ragged rows cross tile boundaries."""
    sizes, offs = expert_offsets(hap, (1.0, 1.0, 0.5, 0.5), 30)
    assert sizes == [10, 10, 5, 5]
    rng = np.random.default_rng(3)
    rows = rng.integers(0, 641, 30); rows[4] = 640; rows[11] = 0
    run_moe_case(hap, "bf16", 30, 640, 512, 1280, offs, rows, act=True, bias=True, full=True)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_moe_unaligned_layout_takes_generic_path(hap, dtype):
    """Odd leading dimensions (no 16-byte rows): the grouped scalar fallback must give the same answers."""
    offs = [0, 2, 3]
    run_moe_case(hap, dtype, 3, 37, 21, 19, offs, [37, 5, 20], act=True, bias=True, full=True, pad=1)
    run_moe_case(hap, dtype, 3, 37, 24, 16, offs, [0, 36, 37], act=False, bias=True, full=False, pad=3)


def test_moe_single_expert_device_equals_linear_layer(hap):
    """A device with one expert and all rows valid is an ordinary fully-connected layer: same bits as hap_sharded_linear_fwd."""
    torch = torch_mod()
    C_, in_f, out_f = 384, 256, 512
    Xh, Xd = gen(2, T.X, (1, C_, in_f), 1.0, "bf16"); Wh, Wd = gen(2, T.W, (1, in_f, out_f), 0.05, "bf16")
    bh, bd = gen(2, T.BIAS, (1, out_f), 0.5, "bf16")
    desc = hap.MoeDesc(1, C_, in_f, out_f, [0, 1], 1, act=1, has_bias=True)
    Y = empty((1, C_, out_f), "bf16", 0); P = empty((1, C_, out_f), "bf16", 0)
    hap.hap_moe_linear_fwd(desc, 0, Xd, Wd, bd, None, Y, P)
    ld = hap.LinearDesc(C_, in_f, out_f, hap.REPLICATED, [0, 1], 1, act=1, has_bias=True, m=1)
    Y2 = empty((C_, out_f), "bf16", 0); P2 = empty((C_, out_f), "bf16", 0)
    hap.hap_sharded_linear_fwd(ld, 0, Xd, Wd, bd, Y2, P2)
    torch.cuda.synchronize()
    assert torch.equal(Y[0], Y2) and torch.equal(P[0], P2)


@pytest.mark.parametrize("fuse_act_bwd", [True, False])
def test_moe_expert_ffn_block_uneven_devices(hap, fuse_act_bwd):
    """Whole expert feed-forward block (fc1 + GeLU + fc2, forward and backward) for 11 experts placed (4, 4, 2, 1) on devices of
    speeds (1, 1, 0.5, 0.3): every device's slice against the unsharded oracle block; with the GeLU backward folded into the
    grouped dH products (the buffer dH then holds dP = dH * gelu'(pre) on the experts' token rows) and as a pass of its own."""
    from oracle import layers as olay, pointwise as opw
    from paper_2401_05965_amd.programs import MoeExpertShard
    torch = torch_mod()
    E, C, Hd, F = 11, 200, 192, 456
    sizes, offs = expert_offsets(hap, (1.0, 1.0, 0.5, 0.3), E)
    assert sizes == [4, 4, 2, 1]
    Xh, Xd = gen(6, T.X, (E, C, Hd), 1.0, "bf16"); dOh, dOd = gen(6, T.DY, (E, C, Hd), 1.0, "bf16")
    W1h, W1d = gen(6, T.W, (E, Hd, F), 0.05, "bf16"); b1h, b1d = gen(6, T.BIAS, (E, F), 0.1, "bf16")
    W2h, W2d = gen(6, T.W2, (E, F, Hd), 0.05, "bf16"); b2h, b2d = gen(6, T.BETA, (E, Hd), 0.1, "bf16")
    rows = np.array([200, 150, 0, 200, 37, 128, 129, 64, 199, 1, 200])
    rows_d = torch.from_numpy(rows.astype(np.int32)).cuda()
    ref = olay.moe_ffn_block(Xh, W1h, b1h, W2h, b2h, dOh, rows)
    ref["dP"] = ref["dH"] * opw.gelu_grad(ref["pre"])
    live = np.arange(C)[None, :] < rows[:, None]
    for j in range(4):
        s = slice(offs[j], offs[j + 1])
        sh = MoeExpertShard(E, C, Hd, F, offs, j, Xd, W1d, b1d, W2d, b2d, rows_d, dOd, fuse_act_bwd=fuse_act_bwd)
        sh.forward(); sh.backward()
        lv = live[s]
        for name, t in (("H", sh.H), ("out", sh.Out), (sh.dH_holds, sh.dH), ("dX", sh.dX)):
            check(f"{name} dev{j}", host(t)[lv], ref[name][s][lv], "bf16")
        for name, t in (("dW1", sh.dW1), ("db1", sh.db1), ("dW2", sh.dW2), ("db2", sh.db2)):
            check(f"{name} dev{j}", host(t), ref[name][s], "bf16")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_moe_few_experts_split_k(hap, dtype):
    """Devices with one expert each and workspace given: outputs have too few tiles to fill the chip, so the contracted axis is
    split over workgroups - also where the token count (known only on the device) leaves some workgroups without any K tile."""
    run_moe_case(hap, dtype, 2, 1024, 256, 384, [0, 1, 2], [700, 130], act=True, bias=True, full=True, fwd_ws=True)
    run_moe_case(hap, dtype, 3, 1024, 512, 128, [0, 1, 3], [0, 1024, 65], act=False, bias=True, full=False, fwd_ws=True, dw_dtype="f32")
