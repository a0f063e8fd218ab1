"""Integer shard sizes and ownership ranges (Sec. 5.1, last paragraph; Sec. 6 parameter slicing).

Rule, restated: scale the ratios by the dimension length, take each to its
nearest integer, and while the total is off, move one unit on the shard whose
size after the move is closest to its fractional target.  Reading of the
unstated details: ties of .5 round up, ties between shards go to the lowest
device index, a size never drops below zero, and sizes are counted in
`granule`-sized units (e.g. one attention head) so a unit is never split.
"""
from __future__ import annotations

import math
from typing import List, Sequence, Tuple


def round_shards(ratios: Sequence[float], dim_len: int, granule: int = 1) -> Tuple[List[int], List[int]]:
    if granule < 1 or dim_len % granule:
        raise ValueError("granule must divide dim_len")
    units = dim_len // granule
    x = [float(r) * float(units) for r in ratios]
    s = [int(math.floor(v + 0.5)) for v in x]
    while sum(s) > units:
        cand = [(abs((s[j] - 1) - x[j]), j) for j in range(len(s)) if s[j] > 0]
        _, j = min(cand)
        s[j] -= 1
    while sum(s) < units:
        cand = [(abs((s[j] + 1) - x[j]), j) for j in range(len(s))]
        _, j = min(cand)
        s[j] += 1
    sizes = [v * granule for v in s]
    offsets = [0]
    for v in sizes:                         # device j owns [sum_{x<j} s_x, sum_{x<=j} s_x)
        offsets.append(offsets[-1] + v)
    return sizes, offsets
