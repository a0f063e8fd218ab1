"""GPU parity: attention slice fwd / bwd and the row / element helpers against the CPU oracle."""
import numpy as np
import pytest

import hapgen
from hapgen import TensorId as T
from oracle import attention as oatt, pointwise as opw

pytestmark = pytest.mark.gpu

from gpu_util import gen, empty, host, check, torch_mod, TOL  # noqa: E402


@pytest.fixture(scope="module")
def hap():
    import paper_2401_05965_amd as h
    return h


def _bshd_to_bhsd(a, B, S, H, D):
    return a.reshape(B, S, H, D).transpose(0, 2, 1, 3)


@pytest.mark.parametrize("B,H,S,D,over_heads,offsets", [
    (2, 5, 300, 128, True, [0, 2, 2, 5]),      # uneven head counts, one empty device; seq spans tiles + ragged tail
    (5, 3, 197, 64, False, [0, 2, 3, 5]),      # ViT-like: batch slices, seq 197, head_dim 64
    (1, 2, 64, 128, True, [0, 2]),             # exactly one tile
    (1, 1, 1, 64, True, [0, 1]),               # degenerate: a single token attends to itself
    (3, 4, 129, 128, True, [0, 1, 4]),         # one query past a 128-query block, one key past two 64-key tiles
    (2, 2, 63, 64, False, [0, 0, 2]),          # shorter than one tile; first device empty
    (1, 3, 513, 64, True, [0, 3]),             # several blocks with a 1-query tail (512 + 1)
    (4, 2, 31, 128, False, [0, 3, 4]),         # fewer queries than one wave holds
    (1, 9, 256, 128, True, [0, 4, 9]),         # exact multiples of the block and tile sizes
    (2, 2, 96, 64, True, [0, 2]),              # the last 64-key tile is exactly half full (its second half is skipped)
    (1, 2, 97, 128, True, [0, 2]),             # ... and one key more: the second half holds a single key
    (2, 1, 32, 128, False, [0, 1, 2]),         # a single half tile
])
def test_attention_slices_fwd_bwd(hap, B, H, S, D, over_heads, offsets):
    torch = torch_mod()
    shp = (B, S, H, D)
    Qh, Qd = gen(3, T.Q, shp, 1.0, "bf16"); Kh, Kd = gen(3, T.K, shp, 1.0, "bf16")
    Vh, Vd = gen(3, T.V, shp, 1.0, "bf16"); dOh, dOd = gen(3, T.DO, shp, 1.0, "bf16")
    desc = hap.AttnDesc(B, H, S, D, over_heads, offsets)
    O = empty(shp, "bf16", 0); lse = empty((B, H, S), "f32", 0)
    dQ = empty(shp, "bf16", 0); dK = empty(shp, "bf16", 0); dV = empty(shp, "bf16", 0)
    ws = empty((max(hap.hap_attn_bwd_workspace(desc, 0), 16),), "u8")
    tr = lambda a: _bshd_to_bhsd(a, B, S, H, D)
    Oo, lseo = oatt.attn_fwd(tr(Qh), tr(Kh), tr(Vh))
    # backward oracle from exact O; the device uses its own bf16 O for D = rowsum(dO * O)
    dQo, dKo, dVo = oatt.attn_bwd(tr(Qh), tr(Kh), tr(Vh), tr(dOh))
    # The bar is max|err| <= 2e-2 * max|ref| per tensor.  Only where the reference is exactly zero (a single key:
    # P = 1, dP == D, so dS = dQ = dK = 0 and a relative metric is undefined) an absolute bound takes its place:
    # the device forms dP and D from bf16 data in different summation orders, which leaves
    # |err dS| <= 2^-8 P (|dP| + |D|), carried through dQ = scale dS K and dK = scale dS^T Q.
    sc = 1.0 / np.sqrt(D)
    zero_floor = {}
    if S == 1:
        dPa = np.abs(np.einsum("bhqd,bhkd->bhqk", tr(dOh), tr(Vh)))
        Da = np.abs((tr(dOh) * Oo).sum(-1))[..., None]
        eS = 2.0 ** -8 * (dPa + Da)
        zero_floor = {"dQ": sc * np.einsum("bhqk,bhkd->bhqd", eS, np.abs(tr(Kh))),
                      "dK": sc * np.einsum("bhqk,bhqd->bhkd", eS, np.abs(tr(Qh)))}
    for j in range(len(offsets) - 1):
        lo, hi = offsets[j], offsets[j + 1]
        O.zero_(); lse.zero_(); dQ.zero_(); dK.zero_(); dV.zero_()
        hap.hap_sharded_attn_fwd(desc, j, Qd, Kd, Vd, O, lse)
        hap.hap_sharded_attn_bwd(desc, j, Qd, Kd, Vd, O, lse, dOd, dQ, dK, dV, ws)
        got = {n: tr(host(t)) for n, t in (("O", O), ("dQ", dQ), ("dK", dK), ("dV", dV))}
        got_lse = host(lse)
        sl = (slice(None), slice(lo, hi)) if over_heads else (slice(lo, hi),)
        mask = np.zeros((B, H), bool); mask[sl] = True
        for n, ref in (("O", Oo), ("dQ", dQo), ("dK", dKo), ("dV", dVo)):
            if hi > lo:
                err = np.abs(got[n][sl] - ref[sl]).max()
                scale_ref = np.abs(ref[sl]).max()
                assert np.isfinite(got[n][sl]).all()
                if scale_ref == 0.0:
                    assert n in zero_floor and err <= zero_floor[n][sl].max(), f"attn shard{j} {n}: |err| {err:.3e} against an all-zero reference"
                    print(f"attn B{B} H{H} S{S} D{D} shard{j} {n}: reference is exactly zero, |err| = {err:.3e}")
                    continue
                print(f"attn B{B} H{H} S{S} D{D} shard{j} {n}: max|err|/max|ref| = {err / scale_ref:.3e}")
                assert err <= TOL["bf16"] * scale_ref, f"attn shard{j} {n}: max|err|/max|ref| = {err / scale_ref:.3e} > {TOL['bf16']:.0e}"
            assert not got[n][~mask].any(), f"{n}: (batch, head) pairs outside the slice were written"
        if hi > lo:
            assert np.abs(got_lse[sl] - lseo[sl]).max() <= 2e-2
        assert not got_lse[~mask].any()


def test_attention_strided_qkv_views(hap):
    """Q, K, V as column blocks of one [tokens x 3*heads*d] buffer (stride_s larger than heads*d)."""
    torch = torch_mod()
    B, H, S, D = 2, 3, 130, 64
    w = 3 * H * D
    allh, alld = gen(5, T.Q, (B * S, w), 1.0, "bf16")
    dOh, dOd = gen(5, T.DO, (B, S, H, D), 1.0, "bf16")
    desc = hap.AttnDesc(B, H, S, D, True, [0, 3], stride_b=S * w, stride_s=w, stride_h=D)
    es = 2
    base = alld.data_ptr()
    Ostr = empty((B * S, w), "bf16", 0)
    lse = empty((B, H, S), "f32", 0)
    hap.hap_sharded_attn_fwd(desc, 0, base, base + H * D * es, base + 2 * H * D * es, Ostr.data_ptr(), lse)
    q, k, v = (allh[:, i * H * D:(i + 1) * H * D].reshape(B, S, H, D).transpose(0, 2, 1, 3) for i in range(3))
    Oo, _ = oatt.attn_fwd(q, k, v)
    got = host(Ostr)[:, :H * D].reshape(B, S, H, D).transpose(0, 2, 1, 3)
    check("strided O", got, Oo, "bf16")
    assert not host(Ostr)[:, H * D:].any()


def test_attention_argument_errors(hap):
    torch = torch_mod()
    t = empty((1, 8, 1, 64), "bf16", 0); lse = empty((8,), "f32", 0)
    with pytest.raises(hap.HapError) as e:
        hap.hap_sharded_attn_fwd(hap.AttnDesc(1, 1, 8, 96, True, [0, 1]), 0, t, t, t, t, lse)
    assert e.value.status == 7
    with pytest.raises(hap.HapError) as e:
        hap.hap_sharded_attn_fwd(hap.AttnDesc(1, 1, 8, 64, True, [0, 2]), 0, t, t, t, t, lse)
    assert e.value.status == 2


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("rows,n", [(37, 2048), (130, 1024), (5, 200), (4099, 768), (9, 201), (3, 8), (21, 1992), (6, 2047)])
def test_layernorm_fwd_bwd(hap, dtype, rows, n):
    xh, xd = gen(2, T.X, (rows, n), 2.0, dtype)
    gh, gd = gen(2, T.GAMMA, (n,), 0.3, dtype); gh = gh + 0  # gamma ~ N(0, .3): exercises the affine part
    bh, bd = gen(2, T.BETA, (n,), 0.3, dtype)
    dyh, dyd = gen(2, T.DY, (rows, n), 1.0, dtype)
    y = empty((rows, n), dtype, 0); mean = empty((rows,), "f32", 0); rstd = empty((rows,), "f32", 0)
    hap.hap_layernorm_fwd(rows, n, {"bf16": 1, "f32": 0}[dtype], xd, gd, bd, y, mean, rstd)
    yo, muo, rso = opw.layernorm_fwd(xh, gh, bh)
    check("ln y", host(y), yo, dtype)
    assert np.abs(host(mean) - muo).max() <= 1e-4 * max(1, np.abs(muo).max())
    assert np.abs(host(rstd) / rso - 1).max() <= 1e-4
    dx = empty((rows, n), dtype, 0); dg = empty((n,), "f32", 0); db = empty((n,), "f32", 0)
    ws = empty((max(hap.hap_layernorm_bwd_workspace(rows, n), 16),), "u8")
    hap.hap_layernorm_bwd(rows, n, {"bf16": 1, "f32": 0}[dtype], xd, gd, mean, rstd, dyd, dx, dg, db, ws)
    dxo, dgo, dbo = opw.layernorm_bwd(xh, gh, dyh)
    check("ln dx", host(dx), dxo, dtype); check("ln dgamma", host(dg), dgo, dtype); check("ln dbeta", host(db), dbo, dtype)
    # with the residual path's gradient added in the same kernel, out of place and in place (dx = dresidual)
    rh, rd = gen(2, T.DO, (rows, n), 1.0, dtype)
    dx2 = empty((rows, n), dtype, 0)
    hap.hap_layernorm_bwd(rows, n, {"bf16": 1, "f32": 0}[dtype], xd, gd, mean, rstd, dyd, dx2, dg, db, ws, dresidual=rd)
    check("ln dx + dres", host(dx2), dxo + rh, dtype); check("ln dgamma", host(dg), dgo, dtype)
    inpl = rd.clone()
    hap.hap_layernorm_bwd(rows, n, {"bf16": 1, "f32": 0}[dtype], xd, gd, mean, rstd, dyd, inpl, dg, db, ws, dresidual=inpl)
    assert (host(inpl) == host(dx2)).all()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_gelu_bwd_add_colsum(hap, dtype):
    torch = torch_mod()
    io = {"bf16": 1, "f32": 0}[dtype]
    for rows, cols, ld in [(300, 520, 520), (77, 137, 141), (1030, 64, 64), (77, 137, 144), (513, 2731, 2736), (5, 3, 8)]:   # incl. ragged widths on aligned pitches
        ph, pd = gen(4, T.X, (rows, ld), 1.5, dtype); dyh, dyd = gen(4, T.DY, (rows, ld), 1.0, dtype)
        out = empty((rows, ld), dtype, 0)
        hap.hap_gelu_bwd(rows, cols, io, pd, ld, dyd, ld, out, ld)
        check("gelu_bwd", host(out)[:, :cols], (dyh * opw.gelu_grad(ph))[:, :cols], dtype)
        assert not host(out)[:, cols:].any()
        bh, bd = gen(4, T.BIAS, (cols,), 1.0, dtype)
        out.zero_()
        hap.hap_add(rows, cols, io, pd, ld, dyd, ld, bd, out, ld)
        check("add", host(out)[:, :cols], (ph + dyh)[:, :cols] + bh, dtype)
        hap.hap_add(rows, cols, io, pd, ld, dyd, ld, None, pd, ld)           # in place, no bias
        check("add in place", host(pd)[:, :cols], (ph + dyh)[:, :cols], dtype)
        s = empty((cols,), "f32", float("nan"))
        ws = empty((max(hap.hap_colsum_workspace(rows, cols), 16),), "u8")
        hap.hap_colsum(rows, cols, io, dyd, ld, s, ws)
        check("colsum", host(s), dyh[:, :cols].sum(0), dtype)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_gelu_bwd_column_range_of_whole_tensors(hap, dtype):
    """GeLU backward on a column range of whole tensors: the three views start a few elements past a 16-byte boundary (the same phase
    in all of them) and run through chunks aligned in the buffers' own address space; columns outside the range stay untouched."""
    io = {"bf16": 1, "f32": 0}[dtype]; esz = {"bf16": 2, "f32": 4}[dtype]
    rows, ld = 203, 1024
    ph, pd = gen(9, T.X, (rows, ld), 1.5, dtype); dyh, dyd = gen(9, T.DY, (rows, ld), 1.0, dtype)
    for off, cols in [(3, 1000), (5, 1019), (1, 7), (2, 520), (6, 1), (8, 333)]:
        if dtype == "f32" and off % 4 == 0 and off:
            continue
        out = empty((rows, ld), dtype, 7)
        hap.hap_gelu_bwd(rows, cols, io, pd.data_ptr() + off * esz, ld, dyd.data_ptr() + off * esz, ld, out.data_ptr() + off * esz, ld)
        got = host(out)
        check("gelu_bwd skewed", got[:, off:off + cols], (dyh * opw.gelu_grad(ph))[:, off:off + cols], dtype)
        assert (got[:, :off] == 7).all() and (got[:, off + cols:] == 7).all()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_colsum_unaligned_base(hap, dtype):
    """Column sums of a view that starts 3 elements into an aligned buffer (vector path with a skew)."""
    io = {"bf16": 1, "f32": 0}[dtype]; esz = {"bf16": 2, "f32": 4}[dtype]
    rows, ld = 333, 1024
    ah, ad = gen(5, T.DY, (rows + 1, ld), 1.0, dtype)
    for off, cols in [(3, 1000), (5, 1019), (1, 7), (8, 520)]:
        s = empty((cols,), "f32", float("nan"))
        ws = empty((max(hap.hap_colsum_workspace(rows, cols), 16),), "u8")
        hap.hap_colsum(rows, cols, io, ad.data_ptr() + off * esz, ld, s, ws)
        check("colsum skew", host(s), ah[:rows, off:off + cols].sum(0), dtype)


def test_row_ops_degenerate_sizes(hap):
    """Empty and one-element extents: every helper returns HAP_OK and leaves what it does not own untouched."""
    for dtype in ("bf16", "f32"):
        io = {"bf16": 1, "f32": 0}[dtype]
        # LayerNorm over a single column: y = beta, dx = 0, dgamma = 0, dbeta = colsum(dy)
        xh, xd = gen(6, T.X, (5, 1), 1.0, dtype); gh, gd = gen(6, T.GAMMA, (1,), 1.0, dtype); bh, bd = gen(6, T.BETA, (1,), 1.0, dtype)
        dyh, dyd = gen(6, T.DY, (5, 1), 1.0, dtype)
        y = empty((5, 1), dtype, 7); mean = empty((5,), "f32", 0); rstd = empty((5,), "f32", 0)
        hap.hap_layernorm_fwd(5, 1, io, xd, gd, bd, y, mean, rstd)
        yo, _, _ = opw.layernorm_fwd(xh, gh, bh)
        check("ln n=1", host(y), yo, dtype)
        dx = empty((5, 1), dtype, 7); dg = empty((1,), "f32", 7); db = empty((1,), "f32", 7)
        ws = empty((max(hap.hap_layernorm_bwd_workspace(5, 1), 16),), "u8")
        hap.hap_layernorm_bwd(5, 1, io, xd, gd, mean, rstd, dyd, dx, dg, db, ws)
        dxo, dgo, dbo = opw.layernorm_bwd(xh, gh, dyh)
        assert np.abs(host(dx) - dxo).max() <= 1e-3 and abs(host(dg)[0] - dgo[0]) <= 1e-2 * max(1.0, np.abs(dyh).sum())
        check("ln n=1 dbeta", host(db), dbo, dtype)
        # zero rows: nothing written except the column sums, which are zero
        s = empty((9,), "f32", float("nan")); keep = empty((4, 9), dtype, 3)
        ws = empty((16,), "u8")
        hap.hap_colsum(0, 9, io, keep, 9, s, ws)
        assert not host(s).any()
        hap.hap_layernorm_fwd(0, 9, io, keep, keep, keep, keep, mean, rstd)
        # LayerNorm backward of an empty shard: dx has no rows, the partial parameter gradients are empty sums = zeros
        dg9 = empty((9,), "f32", float("nan")); db9 = empty((9,), "f32", float("nan"))
        hap.hap_layernorm_bwd(0, 9, io, keep, keep, mean, rstd, keep, keep, dg9, db9, ws)
        assert not host(dg9).any() and not host(db9).any()
        hap.hap_gelu_bwd(0, 9, io, keep, 9, keep, 9, keep, 9)
        hap.hap_add(0, 9, io, keep, 9, keep, 9, None, keep, 9)
        hap.hap_add(4, 0, io, keep, 9, keep, 9, None, keep, 9)
        assert (host(keep) == 3).all()
