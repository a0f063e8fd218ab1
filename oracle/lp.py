"""Sharding-ratio optimisation (Sec. 5.1, Eq. "opt_B"; cost model of Sec. 3.2).

A stage i is described by four numbers, all inputs:
  flops_sharded  F_i  flops whose count scales with the device's ratio B_j
  flops_fixed    G_i  flops every device executes regardless of B_j
  comm_latency   a_i  seconds, constant part of the stage's collective
  comm_per_ratio c_i  seconds per unit of max_j B_j (bytes of the whole tensor / bandwidth)

Per-iteration time (Sec. 3.2):  t(B) = sum_i [ a_i + c_i * max_j B_j + max_j (F_i*B_j + G_i)/s_j ].
The optimiser is the epigraph form of that min-max problem handed to a library
LP routine; it is not a simplex of our own.
"""
from __future__ import annotations

import numpy as np
from scipy.optimize import linprog


def iteration_time(B, speed, stages) -> float:
    """t(Q,B) of Sec. 3.2 for the linear stage model; stages = [(F, G, a, c), ...]."""
    B = np.asarray(B, dtype=np.float64)
    s = np.asarray(speed, dtype=np.float64)
    total = 0.0
    bmax = float(B.max())
    for (F, G, a, c) in stages:
        comp = (F * B + G) / s
        total += a + c * bmax + float(comp.max())
    return total


def shard_ratios(speed, stages):
    """argmin_B t(B) s.t. sum B = 1, B >= 0  (Eq. opt_B).  Returns (B, t(B)).

    Variables: B_1..B_m, u (>= every B_j), t_1..t_S (>= every device's compute time in stage i).
    """
    s = np.asarray(speed, dtype=np.float64)
    m, S = len(s), len(stages)
    nv = m + 1 + S
    cost = np.zeros(nv)
    const = 0.0
    for i, (F, G, a, c) in enumerate(stages):
        cost[m] += c
        cost[m + 1 + i] = 1.0
        const += a
    A_ub, b_ub = [], []
    for j in range(m):                      # B_j - u <= 0
        row = np.zeros(nv); row[j] = 1.0; row[m] = -1.0
        A_ub.append(row); b_ub.append(0.0)
    for i, (F, G, a, c) in enumerate(stages):
        for j in range(m):                  # F/s_j * B_j - t_i <= -G/s_j
            row = np.zeros(nv); row[j] = F / s[j]; row[m + 1 + i] = -1.0
            A_ub.append(row); b_ub.append(-G / s[j])
    A_eq = np.zeros((1, nv)); A_eq[0, :m] = 1.0
    res = linprog(cost, A_ub=np.array(A_ub), b_ub=np.array(b_ub), A_eq=A_eq, b_eq=[1.0],
                  bounds=[(0, None)] * nv, method="highs")
    if res.status != 0:
        raise RuntimeError(f"LP failed: {res.message}")
    B = np.clip(res.x[:m], 0.0, None)
    B = B / B.sum()
    return B, iteration_time(B, s, stages)


def shard_ratios_segments(speed, stages, seg_offsets):
    """Different ratios across the model (Sec. 5.2): stages [seg_offsets[k], seg_offsets[k+1]) form segment k, devices
    synchronise at every boundary (where an All-To-All re-shards), so each segment is Eq. (opt_B) on its own stages.
    Returns (g x m array, total seconds)."""
    o = [int(v) for v in seg_offsets]
    if o[0] != 0 or o[-1] != len(stages) or any(b <= a for a, b in zip(o, o[1:])):
        raise ValueError("segments must be non-empty and cover all stages")
    rows, total = [], 0.0
    for a, b in zip(o, o[1:]):
        B, t = shard_ratios(speed, stages[a:b])
        rows.append(B); total += t
    return np.array(rows), total


def iteration_time_segments(B, speed, stages, seg_offsets) -> float:
    o = [int(v) for v in seg_offsets]
    return sum(iteration_time(B[k], speed, stages[a:b]) for k, (a, b) in enumerate(zip(o, o[1:])))
