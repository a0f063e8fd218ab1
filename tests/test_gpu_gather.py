"""GPU parity of the uneven All-Gather data movement (Sec. 2.3.1: padded slots / grouped pieces -> the full tensor)
against the CPU oracle, through the C ABI.  Byte work: results are compared bit-exactly."""
import numpy as np
import pytest

from oracle import gather as og, lp as olp, rounding as ornd

pytestmark = pytest.mark.gpu

from gpu_util import torch_mod  # noqa: E402

NP = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}


@pytest.fixture(scope="module")
def hap():
    import paper_2401_05965_amd as h
    return h


def pattern(rows, cols, eb):
    v = (np.arange(rows * cols, dtype=np.uint64).reshape(rows, cols) * np.uint64(2654435761) + np.uint64(12345))
    return (v % np.uint64(1 << (8 * min(eb, 4)))).astype(NP[eb])


def dev(a):
    torch = torch_mod()
    return torch.from_numpy(a.view(np.uint8).copy()).cuda()       # device buffers are raw bytes


def back(t, dtype, shape):
    torch = torch_mod()
    torch.cuda.synchronize()
    return t.cpu().numpy().view(dtype).reshape(shape)


def run_case(hap, rows, cols, dim, speeds, eb, ld_extra=0, base_shift=0):
    torch = torch_mod()
    n = rows if dim == 0 else cols
    r, _ = hap.hap_shard_ratios(speeds, [(1.0, 0, 0, 0)])
    sizes, offs = hap.hap_round_shards(r, n, 1)
    assert (sizes, offs) == ornd.round_shards(olp.shard_ratios(speeds, [(1.0, 0, 0, 0)])[0], n, 1)
    full = pattern(rows, cols, eb)
    m = len(sizes)
    desc = hap.GatherDesc(rows, cols, dim, offs, eb)
    cap = hap.hap_allgather_capacity(desc)
    assert cap == max(sizes)
    shards = [np.ascontiguousarray(og.shard(full, offs, j, dim)) for j in range(m)]
    POISON = NP[eb](0xA5)
    # ---- pad: every device's shard into its slot of the padded send / receive buffer (slots pre-filled with poison)
    slot_shape = (cap, cols + ld_extra) if dim == 0 else (rows, cap + ld_extra)
    slots_h = np.full((m,) + slot_shape, POISON, dtype=NP[eb])
    slots = dev(slots_h)
    slot_bytes = slot_shape[0] * slot_shape[1] * eb
    shard_d = [dev(s) if s.size else None for s in shards]
    for j in range(m):
        hap.hap_allgather_pad(desc, j, shard_d[j], shards[j].shape[1], slots.data_ptr() + j * slot_bytes, slot_shape[1])
    got_slots = back(slots, NP[eb], (m,) + slot_shape)
    for j in range(m):
        want = og.pad(shards[j], cap, dim, fill=POISON)
        assert np.array_equal(got_slots[j][:, :want.shape[1]], want), f"pad: slot {j}"
        assert (got_slots[j][:, want.shape[1]:] == POISON).all()
    # ---- trim: the padded slots -> the full tensor, one launch; out has a wider leading dimension and an odd base
    ld_out = cols + ld_extra
    out_raw = dev(np.full((rows * ld_out * eb + 64,), 0x5A, dtype=np.uint8))
    out_ptr = out_raw.data_ptr() + base_shift * eb
    hap.hap_allgather_assemble(desc, [slots.data_ptr() + j * slot_bytes for j in range(m)], [slot_shape[1]] * m, out_ptr, ld_out)
    want_full = og.assemble([got_slots[j][:, :cols] if dim == 0 else got_slots[j] for j in range(m)], offs, dim)
    assert np.array_equal(want_full, full)
    raw = back(out_raw, np.uint8, (-1,))
    got = raw[base_shift * eb: base_shift * eb + rows * ld_out * eb].view(NP[eb]).reshape(rows, ld_out)
    assert np.array_equal(got[:, :cols], full), "trim"
    assert (got[:, cols:].view(np.uint8) == 0x5A).all() and (raw[:base_shift * eb] == 0x5A).all() and (raw[base_shift * eb + rows * ld_out * eb:] == 0x5A).all()
    # ---- grouped layout: every shard at its own size, straight into place
    out2 = dev(np.zeros((rows, cols), dtype=NP[eb]))
    hap.hap_allgather_assemble(desc, shard_d, [max(s.shape[1], 1) for s in shards], out2, cols)
    assert np.array_equal(back(out2, NP[eb], (rows, cols)), og.assemble(shards, offs, dim)), "grouped"
    # ---- the reverse, before a padded Reduce-Scatter: the full tensor (odd base, wide leading dimension) cut into m slots
    # of capacity size, shard range first, zeros behind; bytes past a slot's width keep their poison
    src_raw = dev(np.full((rows * ld_out * eb + 64,), 0x5A, dtype=np.uint8))
    src_h = np.full((rows, ld_out), NP[eb](0x33), dtype=NP[eb]); src_h[:, :cols] = full
    src_raw[base_shift * eb: base_shift * eb + rows * ld_out * eb] = torch.from_numpy(src_h.view(np.uint8).reshape(-1).copy()).cuda()
    rs = dev(np.full((m,) + slot_shape, POISON, dtype=NP[eb]))
    hap.hap_reducescatter_split(desc, src_raw.data_ptr() + base_shift * eb, ld_out, [rs.data_ptr() + j * slot_bytes for j in range(m)],
                                [slot_shape[1]] * m)
    got_rs = back(rs, NP[eb], (m,) + slot_shape)
    want_rs = og.reducescatter_split(full, offs, dim)
    for j in range(m):
        w = want_rs[j].shape[1]
        assert np.array_equal(got_rs[j][:, :w], want_rs[j]), f"reduce-scatter slot {j}"
        assert (got_rs[j][:, w:] == POISON).all()


@pytest.mark.parametrize("eb", [2, 4])
@pytest.mark.parametrize("dim", [0, 1])
def test_gather_aligned(hap, dim, eb):
    """Sizes that keep every address a multiple of 16 bytes (the vector path); 3 devices, uneven."""
    run_case(hap, 640, 1024, dim, (1.0, 0.5, 0.5), eb)


@pytest.mark.parametrize("eb", [1, 2, 4, 8])
@pytest.mark.parametrize("dim", [0, 1])
def test_gather_ragged_everything(hap, dim, eb):
    """Odd shapes, an empty shard, padded leading dimensions and an output base that is only element-aligned."""
    run_case(hap, 203, 77, dim, (1.0, 0.6, 0.35, 0.001), eb, ld_extra=3, base_shift=1)


def test_gather_cfg2_feature_shards_bf16(hap):
    """Config 2's hidden activations, feature-sharded (8402, 5041, 2941) of 16384 columns, at a reduced token count."""
    run_case(hap, 512, 16384, 1, (1.0, 0.6, 0.35), 2)


def test_gather_many_devices(hap):
    run_case(hap, 4099, 40, 0, tuple(1.0 + 0.03 * i for i in range(64)), 2)


def test_gather_cfg2_full_size(hap):
    """The size bench.py times: config 2's [8192 x 16384] bf16 activations from three padded column slots, every byte compared."""
    run_case(hap, 8192, 16384, 1, (1.0, 0.6, 0.35), 2)


@pytest.mark.parametrize("eb", [2, 4])
def test_all_to_all_reshard_from_rows_to_columns(hap, eb):
    """All-To-All at a segment boundary (Sec. 5.2): rows sharded with one set of ratios become columns sharded with another.
    Every virtual device cuts its row shard into m zero-padded column pieces (hap_reducescatter_split on the shard), piece j
    goes to device j, which stacks what arrives by the old row ranges (hap_allgather_assemble).  Bit-exact against the definition."""
    torch = torch_mod()
    rows, cols = 333, 470
    full = pattern(rows, cols, eb)
    r_from, _ = hap.hap_shard_ratios((1.0, 0.6, 0.35, 0.001), [(1.0, 0, 0, 0)])
    r_to, _ = hap.hap_shard_ratios((0.4, 1.0, 0.9, 0.7), [(1.0, 0, 0, 0)])
    _, offs_rows = hap.hap_round_shards(r_from, rows, 1)
    sizes_to, offs_cols = hap.hap_round_shards(r_to, cols, 1)
    m, cap = 4, max(sizes_to)
    shards = [np.ascontiguousarray(og.shard(full, offs_rows, i, 0)) for i in range(m)]
    want = og.all_to_all(shards, offs_rows, 0, offs_cols, 1)
    # send side: device i's pieces, [m][rows_i x cap]
    sent = []
    for i in range(m):
        ri = shards[i].shape[0]
        buf = dev(np.full((m, max(ri, 1), cap), NP[eb](0xA5), dtype=NP[eb]))
        if ri:
            d = hap.GatherDesc(ri, cols, 1, offs_cols, eb)
            hap.hap_reducescatter_split(d, dev(shards[i]), cols, [buf.data_ptr() + j * max(ri, 1) * cap * eb for j in range(m)], [cap] * m)
        sent.append(buf)
    # receive side: device j stacks piece (i -> j) of every i along the rows
    dj = hap.GatherDesc(rows, cap, 0, offs_rows, eb)
    for j in range(m):
        out = dev(np.zeros((rows, cap), dtype=NP[eb]))
        pieces = [sent[i].data_ptr() + j * max(shards[i].shape[0], 1) * cap * eb for i in range(m)]
        hap.hap_allgather_assemble(dj, pieces, [cap] * m, out, cap)
        got = back(out, NP[eb], (rows, cap))
        assert np.array_equal(got[:, :sizes_to[j]], want[j]), f"device {j}"
        assert not got[:, sizes_to[j]:].any()                     # the padding arrives as zeros
