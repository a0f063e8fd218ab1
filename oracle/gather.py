"""All-Gather of an unevenly sharded tensor as one device sees it (Sec. 2.2, Sec. 2.3.1, Fig. "comm_opt").

All-Gather(e, d) concatenates the devices' slices of tensor e along dimension d.  With uneven shard
sizes s_j the collective library wants equal-size pieces, so there are two data layouts:

  padded All-Gather   every device copies its shard into a slot padded to cap = max_j s_j along d
                      ("pad"), the m slots are exchanged, and every device then copies the valid part
                      of each slot to its place in the full tensor ("trim");
  grouped Broadcast   every shard travels at its own size and is put straight into place.

Either way the result is the definition: out[o_j : o_j + s_j] = shard_j along d, o_j = sum_{x<j} s_x.
What the pad region of a slot holds is unspecified (here NaN, so that a read of it shows up).
Any dtype: the movement is exact, tests compare bit patterns.
"""
from __future__ import annotations

import numpy as np


def _offsets(offsets):
    o = [int(v) for v in offsets]
    if o[0] != 0 or any(b < a for a, b in zip(o, o[1:])):
        raise ValueError("offsets must start at 0 and not decrease")
    return o


def shard(full, offsets, j, dim):
    """Device j's slice of the full 2-D tensor along dim."""
    o = _offsets(offsets)
    return full[o[j]:o[j + 1], :] if dim == 0 else full[:, o[j]:o[j + 1]]


def pad(piece, cap, dim, fill=np.nan):
    """The device's send slot: its shard followed by padding up to cap along dim."""
    shape = (cap, piece.shape[1]) if dim == 0 else (piece.shape[0], cap)
    slot = np.full(shape, fill, dtype=piece.dtype)
    if dim == 0:
        slot[:piece.shape[0], :] = piece
    else:
        slot[:, :piece.shape[1]] = piece
    return slot


def assemble(pieces, offsets, dim):
    """out[o_j : o_j + s_j] = pieces[j][: s_j] along dim; pieces may be longer than s_j along dim (padded slots)."""
    o = _offsets(offsets)
    if len(pieces) != len(o) - 1:
        raise ValueError("one piece per device")
    other = pieces[0].shape[1 - dim]
    shape = (o[-1], other) if dim == 0 else (other, o[-1])
    out = np.empty(shape, dtype=pieces[0].dtype)
    for j, p in enumerate(pieces):
        s = o[j + 1] - o[j]
        if dim == 0:
            out[o[j]:o[j + 1], :] = p[:s, :]
        else:
            out[:, o[j]:o[j + 1]] = p[:, :s]
    return out


def reducescatter_split(full, offsets, dim, cap=None):
    """Before a padded Reduce-Scatter (Sec. 2.3.1: the collective needs equal shards): the device's full partial tensor cut
    into m slots of capacity cap = max_j s_j along dim, slot j = the range of shard j followed by ZEROS (they take part in
    the element-wise sums and must not change them).  Returns the list of slots."""
    o = _offsets(offsets)
    sizes = [b - a for a, b in zip(o, o[1:])]
    cap = max(sizes) if cap is None else cap
    return [pad(shard(full, o, j, dim), cap, dim, fill=0) for j in range(len(sizes))]


def all_to_all(shards, offsets_from, dim_from, offsets_to, dim_to):
    """All-To-All(e, d, d') of Sec. 2.2 / Sec. 5.2 as the definition: the devices' slices of e along dim_from (ranges
    offsets_from) become the devices' slices of e along dim_to (ranges offsets_to).  Returns the new list of shards."""
    full = assemble(shards, offsets_from, dim_from)
    return [shard(full, offsets_to, j, dim_to) for j in range(len(_offsets(offsets_to)) - 1)]
