"""GPU parity: sharded linear fwd / bwd and SFB rebuild against the CPU oracle, through the C ABI.

Tolerances (max|err| / max|ref| per output tensor): 1e-5 for fp32, 2e-2 for bf16 inputs with fp32
accumulation; shard index ranges are compared bit-exactly.
"""
import numpy as np
import pytest

import hapgen
from hapgen import TensorId as T
from oracle import linear as olin, sfb as osfb, lp as olp, rounding as ornd

pytestmark = pytest.mark.gpu

from gpu_util import gen, empty, host, check, relerr, torch_mod  # noqa: E402


@pytest.fixture(scope="module")
def hap():
    import paper_2401_05965_amd as h
    return h


DT = {"bf16": 1, "f32": 0}


def run_linear_case(hap, dtype, tokens, in_f, out_f, mode, offsets, act, bias, full, dw_dtype=None, pad=0, seed=7):
    """Runs every shard of one layer on the GPU and checks each against the oracle.  Returns max error."""
    torch = torch_mod()
    dw_dtype = dw_dtype or dtype
    if mode == olin.REDUCTION:
        bias = False          # bias is applied once, after the all-reduce of the partials
    Xh, Xd = gen(seed, T.X, (tokens, in_f), 1.0, dtype)
    Wh, Wd = gen(seed, T.W, (in_f, out_f), 0.05, dtype)
    bh, bd = gen(seed, T.BIAS, (out_f,), 0.5, dtype) if bias else (None, None)
    dYh, dYd = gen(seed, T.DY, (tokens, out_f), 1.0, dtype)
    m = len(offsets) - 1
    worst = 0.0
    Yfull, prefull = olin.linear_fwd(Xh, Wh, bh, act)
    dXsum = np.zeros_like(Xh); dWsum = np.zeros_like(Wh); dbsum = np.zeros(out_f)
    Psum = np.zeros_like(Yfull)
    for j in range(m):
        lo, hi = offsets[j], offsets[j + 1]
        n = hi - lo
        Yo, preo = olin.sharded_linear_fwd(mode, offsets, j, Xh, Wh, bh, act)
        # the oracle's backward takes the full-precision pre-activation; the device uses what it saved
        dXo, dWo, dbo = olin.sharded_linear_bwd(mode, offsets, j, Xh, Wh, prefull if mode != olin.REDUCTION else None, dYh, act)
        if full:
            ldx, ldw, ldy = in_f, out_f, out_f
            Xj, Wj, bj, dYj = Xd, Wd, bd, dYd
            Yj = empty((tokens, out_f), dtype, 0); Pj = empty((tokens, out_f), dtype, 0) if act else None
            dXj = empty((tokens, in_f), dtype, 0); dWj = empty((in_f, out_f), dw_dtype, 0); dbj = empty((out_f,), "f32", 0)
        else:
            # compact slices with padded leading dimensions (pad extra columns filled with NaN poison)
            def compact(t, rows, cols, fill=float("nan")):
                buf = empty((t.shape[0] if rows is None else rows.stop - rows.start, (cols.stop - cols.start if cols else t.shape[1]) + pad), dtype, fill)
                src = t[rows if rows is not None else slice(None), cols if cols is not None else slice(None)]
                buf[:, :src.shape[1]] = src
                return buf
            r = slice(lo, hi)
            if mode == olin.BATCH:
                Xj, Wj, bj, dYj = compact(Xd, r, None), compact(Wd, None, None), bd, compact(dYd, r, None)
                shapeY, shapeX, shapeW = (n, out_f), (n, in_f), (in_f, out_f)
            elif mode == olin.FEATURE:
                Xj, Wj, dYj = compact(Xd, None, None), compact(Wd, None, r), compact(dYd, None, r)
                bj = bd[lo:hi].clone() if bias else None
                shapeY, shapeX, shapeW = (tokens, n), (tokens, in_f), (in_f, n)
            elif mode == olin.REDUCTION:
                Xj, Wj, bj, dYj = compact(Xd, None, r), compact(Wd, r, None), None, compact(dYd, None, None)
                shapeY, shapeX, shapeW = (tokens, out_f), (tokens, n), (n, out_f)
            else:
                Xj, Wj, bj, dYj = compact(Xd, None, None), compact(Wd, None, None), bd, compact(dYd, None, None)
                shapeY, shapeX, shapeW = (tokens, out_f), (tokens, in_f), (in_f, out_f)
            ldx, ldw, ldy = shapeX[1] + pad, shapeW[1] + pad, shapeY[1] + pad
            Yj = empty((shapeY[0], ldy), dtype, 0); Pj = empty((shapeY[0], ldy), dtype, 0) if act else None
            dXj = empty((shapeX[0], ldx), dtype, 0); dWj = empty((shapeW[0], ldw), dw_dtype, 0)
            dbj = empty((shapeY[1],), "f32", 0)
        desc = hap.LinearDesc(tokens, in_f, out_f, mode, offsets, DT[dtype], act=int(act), has_bias=bias and mode != olin.REDUCTION,
                              ldx=ldx, ldw=ldw, ldy=ldy, operands_are_full=full)
        ws = empty((max(hap.hap_linear_bwd_workspace(desc, j), 16),), "u8")
        hap.hap_sharded_linear_fwd(desc, j, Xj, Wj, bj if mode != olin.REDUCTION else None, Yj, Pj, None)
        want_db = mode != olin.REDUCTION
        hap.hap_sharded_linear_bwd(desc, j, Xj, Wj, Pj, dYj, dXj, dWj, DT[dw_dtype], dbj if want_db else None, ws)
        Yg, dXg, dWg, dbg = host(Yj), host(dXj), host(dWj), host(dbj)
        # carve the device's slice out of what came back
        if full:
            if mode == olin.BATCH:
                Ys, dXs, dWs, dbs = Yg[lo:hi], dXg[lo:hi], dWg, dbg
                assert not Yg[:lo].any() and not Yg[hi:].any(), "rows outside the shard were written"
            elif mode == olin.FEATURE:
                Ys, dXs, dWs, dbs = Yg[:, lo:hi], dXg, dWg[:, lo:hi], dbg[lo:hi]
                assert not Yg[:, :lo].any() and not Yg[:, hi:].any(), "columns outside the shard were written"
                assert not dWg[:, :lo].any() and not dWg[:, hi:].any()
            elif mode == olin.REDUCTION:
                Ys, dXs, dWs, dbs = Yg, dXg[:, lo:hi], dWg[lo:hi], None
                assert not dXg[:, :lo].any() and not dXg[:, hi:].any()
                assert not dWg[:lo].any() and not dWg[hi:].any()
            else:
                Ys, dXs, dWs, dbs = Yg, dXg, dWg, dbg
        else:
            Ys, dXs, dWs = Yg[:, :shapeY[1]], dXg[:, :shapeX[1]], dWg[:, :shapeW[1]]
            dbs = dbg if want_db else None
        if n == 0 and mode in (olin.BATCH, olin.FEATURE):
            assert Ys.size == 0 or mode == olin.FEATURE
        tag = f"{dtype} mode{mode} shard{j} full{int(full)}"
        worst = max(worst, check(tag + " Y", Ys, Yo, dtype), check(tag + " dX", dXs, dXo, dtype), check(tag + " dW", dWs, dWo, dw_dtype if dw_dtype == "bf16" else dtype))
        if want_db:
            worst = max(worst, check(tag + " db", dbs, dbo, dtype))
        if mode == olin.REDUCTION:
            Psum += Ys
        if mode == olin.FEATURE:
            dXsum += dXs
        if mode == olin.BATCH:
            dWsum += dWs; dbsum += dbs
    # the rules of Fig. "semantics": partials sum to the unsharded result
    _, dWfull, dbfull = olin.linear_bwd(Xh, Wh, prefull, dYh, act)
    dXfull = olin.linear_bwd(Xh, Wh, prefull, dYh, act)[0]
    big = 4e-2 if dtype == "bf16" else 1e-5
    if mode == olin.REDUCTION:
        assert relerr(Psum, Yfull) <= big
    if mode == olin.FEATURE:
        assert relerr(dXsum, dXfull) <= big
    if mode == olin.BATCH:
        assert relerr(dWsum, dWfull) <= big and relerr(dbsum, dbfull) <= big
    return worst


def test_cfg1_fc_fp32_two_devices(hap):
    """Single fully-connected layer, fp32, batch rows split by the LP ratios of speeds (1, 0.67)."""
    w = hapgen.WORKLOADS["cfg1_fc_f32"]
    d = w.dims
    ratios, _ = hap.hap_shard_ratios(w.speeds, [(1.0, 0, 0, 0)])
    oratios, _ = olp.shard_ratios(w.speeds, [(1.0, 0, 0, 0)])
    assert np.allclose(ratios, oratios, atol=1e-12)
    sizes, offs = hap.hap_round_shards(ratios, d["tokens"])
    osizes, ooffs = ornd.round_shards(oratios, d["tokens"])
    assert sizes == osizes == [38, 26] and offs == ooffs
    # the workload's own scales: X ~ N(0,1), W ~ N(0,0.02), dY ~ N(0,1); seed 0
    torch = torch_mod()
    Xh, Xd = gen(0, T.X, (64, 1024), 1.0, "f32"); Wh, Wd = gen(0, T.W, (1024, 1024), 0.02, "f32"); dYh, dYd = gen(0, T.DY, (64, 1024), 1.0, "f32")
    desc = hap.LinearDesc(64, 1024, 1024, hap.SHARD_BATCH, offs, hap.F32)
    Y = empty((64, 1024), "f32", 0); dX = empty((64, 1024), "f32", 0)
    Xs, dYs = [], []
    for j in range(2):
        dW = empty((1024, 1024), "f32", 0)
        hap.hap_sharded_linear_fwd(desc, j, Xd, Wd, None, Y, None)
        hap.hap_sharded_linear_bwd(desc, j, Xd, Wd, None, dYd, dX, dW, hap.F32, None)
        _, dWo, _ = olin.sharded_linear_bwd(olin.BATCH, offs, j, Xh, Wh, None, dYh)
        check(f"cfg1 dW_{j}", host(dW), dWo, "f32")
        Xs.append(Xd[offs[j]:offs[j + 1]]); dYs.append(dYd[offs[j]:offs[j + 1]])
    Yo, _ = olin.linear_fwd(Xh, Wh); dXo, dWo, _ = olin.linear_bwd(Xh, Wh, None, dYh)
    check("cfg1 Y", host(Y), Yo, "f32"); check("cfg1 dX", host(dX), dXo, "f32")
    # SFB rebuild from the two devices' gathered factors equals the all-reduced gradient
    dW = empty((1024, 1024), "f32", float("nan"))
    hap.hap_sfb_grad(Xs, dYs, sizes, 1024, 1024, 1024, 1024, hap.F32, dW, 1024)
    check("cfg1 SFB dW", host(dW), osfb.sfb_grad([Xh[:38], Xh[38:]], [dYh[:38], dYh[38:]], sizes), "f32")
    check("cfg1 SFB dW vs unsharded", host(dW), dWo, "f32")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("mode", [0, 1, 2, 3])
@pytest.mark.parametrize("full", [True, False])
def test_linear_modes_ragged(hap, dtype, mode, full):
    tokens, in_f, out_f = 300, 264, 520
    dim = {0: tokens, 1: out_f, 2: in_f, 3: 1}[mode]
    offsets = {0: [0, 131, 131, 257, 300], 1: [0, 137, 137, 391, 520], 2: [0, 99, 99, 200, 264], 3: [0, 1]}[mode]
    assert offsets[-1] == dim
    act = mode in (0, 1, 3)
    run_linear_case(hap, dtype, tokens, in_f, out_f, mode, offsets, act=act, bias=True, full=full)


@pytest.mark.parametrize("full", [True, False])
def test_linear_deep_ragged_contractions(hap, full):
    """Contracted ranges that start off the 16-byte grid and span many K tiles: first / last tiles of a range take the
    general tile body (per-chunk validity, zeroing of out-of-range k), the ones between the branch-free one."""
    run_linear_case(hap, "bf16", 260, 1000, 272, 2, [0, 333, 1000], act=False, bias=False, full=full)      # K ranges 333 | 667 of X columns
    run_linear_case(hap, "bf16", 1100, 200, 264, 0, [0, 451, 1100], act=True, bias=True, full=full)        # bwd-weight contracts 451 | 649 rows
    run_linear_case(hap, "bf16", 150, 264, 1210, 1, [0, 603, 1210], act=True, bias=True, full=full)        # bwd-data contracts 603 | 607 columns


def test_linear_unaligned_leading_dimensions_take_the_scalar_kernel(hap):
    # compact slices whose leading dimension is not a multiple of 16 bytes
    run_linear_case(hap, "bf16", 70, 50, 90, 1, [0, 37, 90], act=True, bias=True, full=False, pad=3)
    run_linear_case(hap, "f32", 70, 50, 90, 2, [0, 21, 50], act=False, bias=False, full=False, pad=1)


def test_linear_bf16_fp32_weight_gradient(hap):
    run_linear_case(hap, "bf16", 515, 256, 384, 1, [0, 129, 384], act=True, bias=True, full=True, dw_dtype="f32")


def test_index_ranges_bit_exact_through_identity(hap):
    """An iota tensor pushed through an identity weight: each shard must reproduce exactly its own rows / columns."""
    torch = torch_mod()
    n = 160
    ratios, _ = hap.hap_shard_ratios([1.0, 0.6, 0.35], [(1.0, 0, 0, 0)])
    sizes, offs = hap.hap_round_shards(ratios, n)
    assert (sizes, offs) == ornd.round_shards(olp.shard_ratios([1.0, 0.6, 0.35], [(1.0, 0, 0, 0)])[0], n)
    iota = torch.arange(n * n, dtype=torch.float32, device="cuda").reshape(n, n) % 251   # exact in bf16
    eye = torch.eye(n, dtype=torch.float32, device="cuda")
    for dtype, td in (("f32", torch.float32), ("bf16", torch.bfloat16)):
        X, W = iota.to(td), eye.to(td)
        for mode in (0, 1):
            desc = hap.LinearDesc(n, n, n, mode, offs, DT[dtype])
            for j in range(3):
                Y = empty((n, n), dtype, -1)
                hap.hap_sharded_linear_fwd(desc, j, X, W, None, Y, None)
                got = host(Y); ref = host(X)
                mask = np.zeros((n, n), bool)
                if mode == 0:
                    mask[offs[j]:offs[j + 1], :] = True
                else:
                    mask[:, offs[j]:offs[j + 1]] = True
                assert np.array_equal(got[mask], ref[mask]) and (got[~mask] == -1).all()


def test_sfb_ragged_segments_padding_never_read(hap):
    rows = [70, 0, 33, 128, 1]
    cap, in_f, out_f = 128, 200, 328
    Xh, Xd, dYh, dYd = [], [], [], []
    for i in range(len(rows)):
        a, b = gen(1, T.SFB_X + i, (cap, in_f), 1.0, "bf16"); Xh.append(a); Xd.append(b)
        a, b = gen(1, T.SFB_DY + i, (cap, out_f), 1.0, "bf16"); dYh.append(a); dYd.append(b)
        Xd[i][rows[i]:] = float("nan"); dYd[i][rows[i]:] = float("nan")     # poison the padded All-Gather rows
    ref = osfb.sfb_grad(Xh, dYh, rows)
    dW = empty((in_f, out_f), "f32", float("nan"))
    hap.hap_sfb_grad(Xd, dYd, rows, in_f, out_f, in_f, out_f, hap.BF16, dW, out_f)
    check("sfb", host(dW), ref, "bf16")
    hap.hap_sfb_grad(Xd, dYd, rows, in_f, out_f, in_f, out_f, hap.BF16, dW, out_f, accumulate=True)
    check("sfb accumulate", host(dW), 2 * ref, "bf16")
    # grouped-Broadcast layout: compact factors (cap_i == rows_i), one device only -> plain X^T dY
    dW1 = empty((in_f, out_f), "f32", 0)
    hap.hap_sfb_grad([Xd[3]], [dYd[3]], [128], in_f, out_f, in_f, out_f, hap.BF16, dW1, out_f)
    check("sfb m=1", host(dW1), Xh[3].T @ dYh[3], "bf16")
    # all devices empty -> zeros
    hap.hap_sfb_grad(Xd, dYd, [0] * 5, in_f, out_f, in_f, out_f, hap.BF16, dW1, out_f)
    assert not host(dW1).any()


def test_sfb_split_k_over_segment_boundaries(hap):
    """With workspace the engine splits the contracted axis over idle compute units; the split points fall
    inside and between the devices' ragged segments.  Result must equal the one-pass result."""
    rows = [300, 0, 77, 512, 130]
    cap, in_f, out_f = 512, 264, 392
    Xh, Xd, dYh, dYd = [], [], [], []
    for i in range(len(rows)):
        a, b = gen(9, T.SFB_X + i, (cap, in_f), 1.0, "bf16"); Xh.append(a); Xd.append(b)
        a, b = gen(9, T.SFB_DY + i, (cap, out_f), 1.0, "bf16"); dYh.append(a); dYd.append(b)
        Xd[i][rows[i]:] = float("nan"); dYd[i][rows[i]:] = float("nan")
    ref = osfb.sfb_grad(Xh, dYh, rows)
    ws = empty((hap.hap_sfb_workspace(len(rows), rows, in_f, out_f),), "u8")
    dW = empty((in_f, out_f), "f32", float("nan"))
    hap.hap_sfb_grad(Xd, dYd, rows, in_f, out_f, in_f, out_f, hap.BF16, dW, out_f, ws=ws)
    check("sfb split-k", host(dW), ref, "bf16")
    dW1 = empty((in_f, out_f), "f32", float("nan"))
    hap.hap_sfb_grad(Xd, dYd, rows, in_f, out_f, in_f, out_f, hap.BF16, dW1, out_f)
    assert np.abs(host(dW1) - host(dW)).max() <= 1e-5 * np.abs(ref).max()      # fp32 partial sums, different order only
    hap.hap_sfb_grad(Xd, dYd, rows, in_f, out_f, in_f, out_f, hap.BF16, dW, out_f, accumulate=True, ws=ws)
    check("sfb split-k accumulate", host(dW), 2 * ref, "bf16")


def test_linear_split_k_with_bias_gelu_and_ragged_view(hap):
    """Deep contraction, few output tiles, bias + GeLU + saved pre-activation, misaligned column range:
    the forward goes through split-K when given workspace."""
    tokens, in_f, out_f = 200, 1024, 520
    offs = [0, 137, 391, 520]
    Xh, Xd = gen(5, T.X, (tokens, in_f), 1.0, "bf16"); Wh, Wd = gen(5, T.W, (in_f, out_f), 0.05, "bf16")
    bh, bd = gen(5, T.BIAS, (out_f,), 0.5, "bf16")
    desc = hap.LinearDesc(tokens, in_f, out_f, hap.SHARD_FEATURE, offs, hap.BF16, act=hap.ACT_GELU_ERF, has_bias=True)
    ws = empty((hap.lib.hap_linear_fwd_workspace(None, 0),), "u8")
    Yo, preo = olin.linear_fwd(Xh, Wh, bh, True)
    Y = empty((tokens, out_f), "bf16", 0); P = empty((tokens, out_f), "bf16", 0)
    for j in range(3):
        hap.hap_sharded_linear_fwd(desc, j, Xd, Wd, bd, Y, P, ws)
    check("split-k Y", host(Y), Yo, "bf16"); check("split-k preact", host(P), preo, "bf16")


def test_cfg1_fp32_split_k_with_workspace(hap):
    """Config 1 again with workspace: 16 output tiles cannot occupy the chip, so the fp32 kernel splits its 16 K tiles
    over more workgroups (fp32 partial tiles + reduction); same 1e-5 bar, forward with bias + GeLU and both gradients."""
    offs = [0, 38, 64]
    Xh, Xd = gen(0, T.X, (64, 1024), 1.0, "f32"); Wh, Wd = gen(0, T.W, (1024, 1024), 0.02, "f32"); dYh, dYd = gen(0, T.DY, (64, 1024), 1.0, "f32")
    bh, bd = gen(0, T.BIAS, (1024,), 0.5, "f32")
    desc = hap.LinearDesc(64, 1024, 1024, hap.SHARD_BATCH, offs, hap.F32, act=hap.ACT_GELU_ERF, has_bias=True)
    Y = empty((64, 1024), "f32", 0); P = empty((64, 1024), "f32", 0); dX = empty((64, 1024), "f32", 0); db = empty((1024,), "f32", 0)
    wsf = empty((hap.lib.hap_linear_fwd_workspace(None, 0),), "u8")
    Yo, Po = olin.linear_fwd(Xh, Wh, bh, True)
    dW_sum = np.zeros((1024, 1024)); db_sum = np.zeros(1024)
    for j in range(2):
        hap.hap_sharded_linear_fwd(desc, j, Xd, Wd, bd, Y, P, wsf)
        wsb = empty((hap.hap_linear_bwd_workspace(desc, j),), "u8")
        dW = empty((1024, 1024), "f32", float("nan"))
        hap.hap_sharded_linear_bwd(desc, j, Xd, Wd, P, dYd, dX, dW, hap.F32, db, wsb)
        dW_sum += host(dW); db_sum += host(db)
    dXo, dWo, dbo = olin.linear_bwd(Xh, Wh, Po, dYh, act=True)
    check("cfg1 split-k Y", host(Y), Yo, "f32"); check("cfg1 split-k preact", host(P), Po, "f32")
    check("cfg1 split-k dX", host(dX), dXo, "f32"); check("cfg1 split-k dW", dW_sum, dWo, "f32"); check("cfg1 split-k db", db_sum, dbo, "f32")


def test_linear_seeded_random_sweep(hap):
    """A seeded sweep over shapes, rules, layouts and options nobody hand-picked: tiny to multi-tile extents, ragged everything,
    random shard boundaries (including empty shards), compact and whole-tensor operands, odd pads."""
    rng = np.random.default_rng(20240105)
    for trial in range(28):
        dtype = "bf16" if trial % 3 else "f32"
        tokens = int(rng.choice([1, 7, 33, 130, 257, 515, 700]))
        in_f = int(rng.choice([1, 8, 24, 100, 264, 513]))
        out_f = int(rng.choice([1, 8, 40, 136, 300, 520]))
        mode = int(rng.choice([olin.BATCH, olin.FEATURE, olin.REDUCTION, olin.REPLICATED]))
        axis = {olin.BATCH: tokens, olin.FEATURE: out_f, olin.REDUCTION: in_f, olin.REPLICATED: 1}[mode]
        m = int(rng.integers(1, 4))
        cuts = sorted(int(c) for c in rng.integers(0, axis + 1, m - 1))
        offsets = [0] + cuts + [axis] if mode != olin.REPLICATED else [0, 1]
        act = bool(rng.integers(0, 2)) and mode != olin.REDUCTION
        bias = bool(rng.integers(0, 2))
        full = bool(rng.integers(0, 2))
        pad = int(rng.choice([0, 0, 1, 8])) if not full else 0
        dw_dtype = "f32" if (dtype == "f32" or rng.integers(0, 2)) else "bf16"
        run_linear_case(hap, dtype, tokens, in_f, out_f, mode, offsets, act, bias, full, dw_dtype=dw_dtype, pad=pad, seed=100 + trial)


def test_cfg1_step_replays_from_a_hip_graph(hap):
    """The library's calls only launch kernels on the given stream (no allocation, no memset, no host synchronisation), so a
    whole latency-bound step - config 1: forward + backward of both devices and the SFB rebuild - can be captured once and
    replayed.  Every replay, with eager work and synchronisations in between, must reproduce the eager results bit for bit."""
    torch = torch_mod()
    offs = [0, 38, 64]
    _, Xd = gen(0, T.X, (64, 1024), 1.0, "f32"); _, Wd = gen(0, T.W, (1024, 1024), 0.02, "f32"); _, dYd = gen(0, T.DY, (64, 1024), 1.0, "f32")
    desc = hap.LinearDesc(64, 1024, 1024, hap.SHARD_BATCH, offs, hap.F32)
    ws = empty((hap.hap_linear_bwd_workspace(desc, 0),), "u8")
    out = {k: empty(s, "f32", 0) for k, s in (("Y", (64, 1024)), ("dX", (64, 1024)), ("dW0", (1024, 1024)), ("dW1", (1024, 1024)), ("dWs", (1024, 1024)))}

    def step():
        for j in range(2):
            hap.hap_sharded_linear_fwd(desc, j, Xd, Wd, None, out["Y"], None, ws)
            hap.hap_sharded_linear_bwd(desc, j, Xd, Wd, None, dYd, out["dX"], out[f"dW{j}"], hap.F32, None, ws)
        hap.hap_sfb_grad([Xd[:38], Xd[38:]], [dYd[:38], dYd[38:]], [38, 26], 1024, 1024, 1024, 1024, hap.F32, out["dWs"], 1024, ws=ws)
    step()
    torch.cuda.synchronize()
    want = {k: v.clone() for k, v in out.items()}
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        step()                      # warm the capture stream's state
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for rep in range(3):
        for v in out.values():
            v.fill_(float(rep + 1))                      # eager work between replays: results must come from the replay
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in out:
            assert torch.equal(out[k], want[k]), (rep, k)
        step()                                           # and an eager step in between
        torch.cuda.synchronize()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("mode,full", [("batch", True), ("batch", False), ("reduction", True), ("reduction", False), ("replicated", False)])
@pytest.mark.parametrize("shape", [(300, 200, 130), (64, 96, 4200), (1031, 517, 263)])
def test_linear_bwd_with_producer_activation_backward(hap, dtype, mode, full, shape):
    """hap_sharded_linear_bwd_dact: dX * gelu'(x_preact) in the dX product's epilogue equals the oracle's dX times the oracle's
    gelu', for every shard of the modes whose dX is complete on the device; shapes take the tiled kernels, the split
    contraction (64 x 96 outputs over 4200) and ragged tiles with odd leading dimensions (the element-wise stores)."""
    from oracle import pointwise as opw
    tokens, in_f, out_f = shape
    code = {"batch": olin.BATCH, "reduction": olin.REDUCTION, "replicated": olin.REPLICATED}[mode]
    axis = {"batch": tokens, "reduction": in_f, "replicated": 1}[mode]
    offsets = [0, axis * 2 // 5, axis * 2 // 5, axis] if mode != "replicated" else [0, 1]
    Xh, Xd = gen(11, T.X, (tokens, in_f), 1.0, dtype); Wh, Wd = gen(11, T.W, (in_f, out_f), 0.05, dtype)
    dYh, dYd = gen(11, T.DY, (tokens, out_f), 1.0, dtype); Ph, Pd = gen(11, T.MISC, (tokens, in_f), 1.5, dtype)   # the producer's pre-activation
    for j in range(len(offsets) - 1):
        lo, hi = offsets[j], offsets[j + 1]
        dXo, dWo, _ = olin.sharded_linear_bwd(code, offsets, j, Xh, Wh, None, dYh, False)
        rs = slice(lo, hi) if mode == "batch" else slice(None)
        cs = slice(lo, hi) if mode == "reduction" else slice(None)
        want = dXo * opw.gelu_grad(Ph[rs, cs])
        if full or mode == "replicated":
            Xj, Wj, dYj, Pj = Xd, Wd, dYd, Pd
            ldx, ldw, ldy = in_f, out_f, out_f
            dXj = empty((tokens, in_f), dtype, float("nan"))
        else:
            Xj, Pj = Xd[rs, cs].contiguous(), Pd[rs, cs].contiguous()
            Wj = Wd[cs].contiguous() if mode == "reduction" else Wd
            dYj = dYd[rs].contiguous()
            ldx, ldw, ldy = Xj.shape[1], out_f, out_f
            dXj = empty(tuple(Xj.shape), dtype, float("nan"))
        if Xj.numel() == 0:
            Xj = Pj = dXj = empty((8, max(ldx, 8)), dtype, 0); ldx = max(ldx, 8)
        desc = hap.LinearDesc(tokens, in_f, out_f, code, offsets, DT[dtype], ldx=ldx, ldw=ldw, ldy=ldy, operands_are_full=full, m=len(offsets) - 1)
        ws = empty((max(hap.hap_linear_bwd_workspace(desc, j), 16),), "u8")
        dWj = empty((Wj.shape[0], ldw), "f32", 0)
        hap.hap_sharded_linear_bwd_dact(desc, j, Xj, Wj, None, dYj, dXj, dWj, hap.F32, None, Pj, hap.ACT_GELU_ERF, ws)
        got = host(dXj)
        if full and mode != "replicated":
            inside = got[rs, cs]
            outside = np.ones(got.shape, bool); outside[rs, cs] = False
            assert np.isnan(got[outside]).all(), "elements outside the shard were written"
            got = inside
        elif hi == lo and mode != "replicated":
            continue
        if want.size:
            e = check(f"{dtype} {mode} full{int(full)} shard {j} dX*gelu'", got, want, dtype)
            # and it is the two-step result: the plain backward followed by the element-wise pass, same roundings
            dX2 = empty(tuple(dXj.shape), dtype, float("nan"))
            hap.hap_sharded_linear_bwd(desc, j, Xj, Wj, None, dYj, dX2, None, hap.F32, None, ws)
            if full and mode != "replicated":
                v2, vp = dX2[rs, cs].contiguous(), Pd[rs, cs].contiguous()
            else:
                v2, vp = dX2, Pj
            two = empty(tuple(v2.shape), dtype, 0)
            hap.hap_gelu_bwd(v2.shape[0], v2.shape[1], DT[dtype], vp, vp.stride(0), v2, v2.stride(0), two, two.stride(0))
            assert relerr(got, host(two)) <= (1e-2 if dtype == "bf16" else 1e-5)


def test_linear_bwd_dact_rejects_partial_sums(hap):
    """In feature mode dX is a partial sum: an activation backward applied before the All-Reduce would be wrong, so the call refuses."""
    desc = hap.LinearDesc(64, 32, 48, olin.FEATURE, [0, 20, 48], hap.F32, ldx=32, ldw=48, ldy=48, operands_are_full=True)
    X, W, dY, dX, P = (empty(s, "f32", 0) for s in ((64, 32), (32, 48), (64, 48), (64, 32), (64, 32)))
    ws = empty((hap.hap_linear_bwd_workspace(desc, 0),), "u8")
    with pytest.raises(hap.HapError):
        hap.hap_sharded_linear_bwd_dact(desc, 0, X, W, None, dY, dX, None, hap.F32, None, P, hap.ACT_GELU_ERF, ws)
    with pytest.raises(hap.HapError):
        d2 = hap.LinearDesc(64, 32, 48, olin.BATCH, [0, 20, 64], hap.F32, ldx=32, ldw=48, ldy=48, operands_are_full=True)
        hap.hap_sharded_linear_bwd_dact(d2, 0, X, W, None, dY, dX, None, hap.F32, None, None, hap.ACT_GELU_ERF, ws)


@pytest.mark.parametrize("tokens", [1, 16, 38, 64])
@pytest.mark.parametrize("in_f,out_f", [(1024, 1024), (256, 1000), (4100, 17), (2048, 8000)])
def test_fp32_layer_with_few_rows(hap, tokens, in_f, out_f):
    """fp32 layers of at most 64 rows (config 1's shards are 38 and 26 rows) run forward and bwd-data in a kernel that splits the
    contraction over the waves of a workgroup and sums the partial tiles through LDS: all row-block counts, ragged column tiles,
    contractions that do not divide by the 16 waves, bias + GeLU + saved pre-activation, and dX through the K-contiguous weight.
    (8000 columns are 125 tiles of 64: just below where the tiled kernel takes over.)"""
    Xh, Xd = gen(3, T.X, (tokens, in_f), 1.0, "f32"); Wh, Wd = gen(3, T.W, (in_f, out_f), 0.05, "f32")
    bh, bd = gen(3, T.BIAS, (out_f,), 0.5, "f32"); dYh, dYd = gen(3, T.DY, (tokens, out_f), 1.0, "f32")
    desc = hap.LinearDesc(tokens, in_f, out_f, olin.REPLICATED, [0, 1], hap.F32, act=hap.ACT_GELU_ERF, has_bias=True, m=1)
    Y = empty((tokens, out_f), "f32", float("nan")); P = empty((tokens, out_f), "f32", float("nan"))
    ws = empty((max(hap.hap_linear_bwd_workspace(desc, 0), 16),), "u8")
    hap.hap_sharded_linear_fwd(desc, 0, Xd, Wd, bd, Y, P, ws)
    Yo, preo = olin.linear_fwd(Xh, Wh, bh, True)
    check("Y", host(Y), Yo, "f32"); check("preact", host(P), preo, "f32")
    dX = empty((tokens, in_f), "f32", float("nan")); dW = empty((in_f, out_f), "f32", float("nan")); db = empty((out_f,), "f32", float("nan"))
    hap.hap_sharded_linear_bwd(desc, 0, Xd, Wd, P, dYd, dX, dW, hap.F32, db, ws)
    dXo, dWo, dbo = olin.linear_bwd(Xh, Wh, preo, dYh, True)
    check("dX", host(dX), dXo, "f32"); check("dW", host(dW), dWo, "f32"); check("db", host(db), dbo, "f32")
