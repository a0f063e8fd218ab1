"""Pins for oracle.gather (Sec. 2.2: All-Gather concatenates the slices along d; Sec. 2.3.1: padded vs grouped)."""
import numpy as np
import pytest

from oracle import gather, lp, rounding


def _full(rows, cols, dtype=np.uint16):
    return (np.arange(rows * cols, dtype=np.int64).reshape(rows, cols) * 2654435761 % 65521).astype(dtype)


@pytest.mark.parametrize("dim", [0, 1])
def test_gather_of_the_shards_is_the_tensor_both_layouts(dim):
    """Slicing a tensor by the LP + rounding ranges and gathering the slices back - through padded slots or at their own
    sizes - is the identity (the definition of All-Gather), for a placement with an empty shard."""
    full = _full(23, 31)
    n = full.shape[dim]
    ratios, _ = lp.shard_ratios((1.0, 0.6, 0.35, 0.001), [(1.0, 0, 0, 0)])
    sizes, offs = rounding.round_shards(ratios, n, 1)
    assert sum(sizes) == n and sizes[-1] == 0
    shards = [gather.shard(full, offs, j, dim) for j in range(4)]
    assert [s.shape[dim] for s in shards] == sizes
    cap = max(sizes)
    slots = [gather.pad(s.astype(np.float64), cap, dim) for s in shards]           # NaN padding: a read of it would show
    assert all(s.shape[dim] == cap for s in slots)
    assert np.array_equal(gather.assemble(slots, offs, dim), full.astype(np.float64))
    assert np.array_equal(gather.assemble(shards, offs, dim), full)
    assert np.array_equal(gather.assemble(shards, offs, dim), np.concatenate(shards, axis=dim))


def test_elementwise_placement_brute_force():
    full = _full(7, 5)
    offs = [0, 3, 3, 7]
    out = gather.assemble([gather.pad(gather.shard(full, offs, j, 0), 4, 0, fill=9) for j in range(3)], offs, 0)
    for r in range(7):
        j = 0 if r < 3 else 2
        for c in range(5):
            assert out[r, c] == full[r, c] == gather.shard(full, offs, j, 0)[r - offs[j], c]
    offs = [0, 1, 5]
    out = gather.assemble([gather.pad(gather.shard(full, offs, j, 1), 4, 1, fill=9) for j in range(2)], offs, 1)
    for r in range(7):
        for c in range(5):
            j = 0 if c < 1 else 1
            assert out[r, c] == gather.shard(full, offs, j, 1)[r, c - offs[j]]


def test_bad_offsets_rejected():
    with pytest.raises(ValueError):
        gather.assemble([_full(2, 2)], [1, 3], 0)
    with pytest.raises(ValueError):
        gather.assemble([_full(2, 2)], [0, 2, 4], 0)


@pytest.mark.parametrize("dim", [0, 1])
def test_reducescatter_slots_brute_force_and_round_trip(dim):
    """Slot j holds the range of shard j, then zeros up to the capacity; putting the slots' valid parts back gives the tensor."""
    full = _full(7, 6)
    offs = [0, 3, 3, 7] if dim == 0 else [0, 1, 1, 6]
    sizes = [b - a for a, b in zip(offs, offs[1:])]
    cap = max(sizes)
    slots = gather.reducescatter_split(full, offs, dim)
    assert len(slots) == 3
    for j, s in enumerate(slots):
        assert s.shape == ((cap, 6) if dim == 0 else (7, cap)) and s.dtype == full.dtype
        for r in range(s.shape[0]):
            for c in range(s.shape[1]):
                k = r if dim == 0 else c                                  # position along the sharded axis
                want = (full[offs[j] + r, c] if dim == 0 else full[r, offs[j] + c]) if k < sizes[j] else 0
                assert s[r, c] == want
    assert not slots[1].any()                                             # the empty shard's slot is all zeros
    assert np.array_equal(gather.assemble(slots, offs, dim), full)


@pytest.mark.parametrize("dim", [0, 1])
def test_padded_reduce_scatter_equals_shard_of_the_sum(dim):
    """What the padding must guarantee: summing slot j over the devices (the collective's reduction) and trimming it gives
    shard j of the summed tensor, and the padding sums to exactly zero - for LP + rounding ranges over unequal devices."""
    rng = np.random.default_rng(4)
    parts = [rng.integers(-50, 50, (12, 10)).astype(np.float64) for _ in range(3)]          # three devices' partial tensors
    n = parts[0].shape[dim]
    ratios, _ = lp.shard_ratios((1.0, 0.6, 0.35), [(1.0, 0, 0, 0)])
    sizes, offs = rounding.round_shards(ratios, n, 1)
    cap = max(sizes)
    total = sum(parts)
    for j in range(3):
        reduced = sum(gather.reducescatter_split(p, offs, dim)[j] for p in parts)               # the slot device j ends up with
        valid = reduced[:sizes[j]] if dim == 0 else reduced[:, :sizes[j]]
        rest = reduced[sizes[j]:] if dim == 0 else reduced[:, sizes[j]:]
        assert np.array_equal(valid, gather.shard(total, offs, j, dim)) and not rest.any()
        assert reduced.shape[dim] == cap


def test_all_to_all_is_split_exchange_assemble():
    """All-To-All(e, 0, 1) re-shards a row-sharded tensor by columns (the segment boundary of Sec. 5.2, with different
    ratios on the two sides).  Its definition must equal the movement a device actually performs: cut the own row shard into m
    column pieces (zero-padded to the new capacity), hand piece j to device j, stack what arrives by the old row ranges."""
    full = _full(11, 9)
    offs_rows, offs_cols = [0, 5, 5, 11], [0, 2, 6, 9]
    m = 3
    shards = [gather.shard(full, offs_rows, i, 0) for i in range(m)]
    want = gather.all_to_all(shards, offs_rows, 0, offs_cols, 1)
    for j in range(m):
        assert np.array_equal(want[j], full[:, offs_cols[j]:offs_cols[j + 1]])
    sent = [gather.reducescatter_split(shards[i], offs_cols, 1) for i in range(m)]       # sent[i][j]: device i's piece for device j
    cap = max(b - a for a, b in zip(offs_cols, offs_cols[1:]))
    for j in range(m):
        got = gather.assemble([sent[i][j] for i in range(m)], offs_rows, 0)               # [11 x cap], valid columns first
        assert got.shape == (11, cap)
        assert np.array_equal(got[:, :offs_cols[j + 1] - offs_cols[j]], want[j])
