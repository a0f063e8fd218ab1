"""Pins for oracle.lp and oracle.rounding (Sec. 2.4, Sec. 3.2, Sec. 5.1, Sec. 6)."""
import itertools
import os

import numpy as np
import pytest

from oracle import lp, rounding

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _lines(name):
    with open(os.path.join(GOLD, name)) as f:
        return [l.strip() for l in f if l.strip() and not l.startswith("#")]


def test_iteration_time_matches_hand_worked_values():
    for l in _lines("lp_worked.txt"):
        if l.startswith("opt"):
            continue
        b1, b2, t = map(float, l.split())
        assert lp.iteration_time([b1, b2], [2.0, 1.0], [(6.0, 0.0, 0.5, 1.0)]) == pytest.approx(t, abs=1e-12)


def test_optimum_matches_hand_worked_closed_form():
    l = [x for x in _lines("lp_worked.txt") if x.startswith("opt")][0].split()
    B, t = lp.shard_ratios([2.0, 1.0], [(6.0, 0.0, 0.5, 1.0)])
    assert B == pytest.approx([float(l[1]), float(l[2])], abs=1e-9)
    assert t == pytest.approx(float(l[3]), abs=1e-9)


@pytest.mark.parametrize("speed", [(1.0, 0.67), (1.0, 0.6, 0.35), (1, 1, .5, .5), (1, .8, .8, .4, .25), (3, 1, 4, 1, 5, 9, 2, 6)])
def test_compute_only_is_proportional_to_speed(speed):
    # Sec. 2.4: with computation only, ratios proportional to device speed are optimal (and unique)
    B, t = lp.shard_ratios(speed, [(7.0e9, 0.0, 0.0, 0.0)])
    s = np.asarray(speed, float)
    assert B == pytest.approx(s / s.sum(), abs=1e-9)
    assert t == pytest.approx(7.0e9 / s.sum(), rel=1e-9)


@pytest.mark.parametrize("m", [2, 3, 5])
def test_communication_only_is_even(m):
    # Sec. 2.4: communication time depends on the largest shard, minimal for the even split
    speed = np.linspace(1.0, 2.0, m)
    B, t = lp.shard_ratios(speed, [(0.0, 0.0, 1e-3, 0.25)])
    assert B == pytest.approx(np.full(m, 1.0 / m), abs=1e-9)
    assert t == pytest.approx(1e-3 + 0.25 / m, rel=1e-9)


@pytest.mark.parametrize("c,expect_even", [(10.0, True), (0.5, False)])
def test_two_devices_single_stage_endpoint(c, expect_even):
    # between the even split and the speed-proportional split t is linear in B_1 with slope c - F/s_slow
    s = (2.0, 1.0); F = 3.0
    B, _ = lp.shard_ratios(s, [(F, 0.0, 0.0, c)])
    assert (c > F / s[1]) == expect_even
    want = [0.5, 0.5] if expect_even else [2 / 3, 1 / 3]
    assert B == pytest.approx(want, abs=1e-9)


def test_mixed_optimum_lies_between_even_and_proportional():
    s = np.array([1.0, 0.6, 0.35])
    stages = [(4.0, 0.3, 1e-3, 2.0), (1.0, 0.0, 2e-3, 0.1), (9.0, 1.0, 0.0, 5.0)]
    B, t = lp.shard_ratios(s, stages)
    assert B.sum() == pytest.approx(1.0, abs=1e-12) and (B >= 0).all()
    assert t <= lp.iteration_time(s / s.sum(), s, stages) + 1e-12
    assert t <= lp.iteration_time(np.full(3, 1 / 3), s, stages) + 1e-12


def test_grid_brute_force_two_and_three_devices():
    rng = np.random.default_rng(5)
    for trial in range(6):
        m = 2 + trial % 2
        s = rng.uniform(0.3, 2.0, m)
        stages = [tuple(rng.uniform(0, 3, 4)) for _ in range(1 + trial % 3)]
        B, t = lp.shard_ratios(s, stages)
        n = 2000 if m == 2 else 150
        best = np.inf
        for idx in itertools.product(range(n + 1), repeat=m - 1):
            if sum(idx) > n:
                continue
            cand = np.array(list(idx) + [n - sum(idx)], float) / n
            best = min(best, lp.iteration_time(cand, s, stages))
        # the grid cannot beat the LP optimum; it comes within the grid's resolution of it
        lipschitz = sum(st[3] + st[0] / s.min() for st in stages)
        assert t <= best + 1e-9
        assert best - t <= lipschitz * (m / n)


def test_invariances():
    s = np.array([1.0, 0.8, 0.8, 0.4, 0.25]); stages = [(5.0, 0.5, 1e-3, 1.0)]
    B, t = lp.shard_ratios(s, stages)
    B2, t2 = lp.shard_ratios(s[::-1], stages)
    assert t2 == pytest.approx(t, rel=1e-9)
    # scaling every speed and the flop counts together leaves the problem unchanged
    B3, t3 = lp.shard_ratios(3 * s, [(15.0, 1.5, 1e-3, 1.0)])
    assert t3 == pytest.approx(t, rel=1e-9)


# ---------------- rounding ----------------

def test_rounding_worked_examples():
    for l in _lines("rounding_worked.txt"):
        n, g, sp, want = [x.strip() for x in l.split("|")]
        sp = np.array(sp.split(), float)
        sizes, offs = rounding.round_shards(sp / sp.sum(), int(n), int(g))
        assert sizes == [int(v) for v in want.split()], l
        assert offs[0] == 0 and offs[-1] == int(n)


def _compositions(total, parts):
    if parts == 1:
        yield (total,)
        return
    for a in range(total + 1):
        for rest in _compositions(total - a, parts - 1):
            yield (a,) + rest


def test_rounding_minimises_l1_error_brute_force():
    rng = np.random.default_rng(11)
    for _ in range(60):
        m = int(rng.integers(2, 5)); n = int(rng.integers(1, 13))
        r = rng.dirichlet(np.ones(m))
        sizes, offs = rounding.round_shards(r, n)
        assert sum(sizes) == n and min(sizes) >= 0
        x = r * n
        best = min(sum(abs(c[j] - x[j]) for j in range(m)) for c in _compositions(n, m))
        assert sum(abs(sizes[j] - x[j]) for j in range(m)) <= best + 1e-9
        assert all(abs(sizes[j] - x[j]) < 1 + 1e-12 for j in range(m))


def test_rounding_integral_targets_exact_and_ranges_tile():
    sizes, offs = rounding.round_shards([0.25, 0.5, 0.0, 0.25], 64)
    assert sizes == [16, 32, 0, 16] and offs == [0, 16, 48, 48, 64]
    covered = []
    for j in range(4):
        covered += list(range(offs[j], offs[j + 1]))
    assert covered == list(range(64))


def test_rounding_granule():
    sizes, offs = rounding.round_shards([1 / 3, 1 / 3, 1 / 6, 1 / 6], 2048, 128)
    assert all(s % 128 == 0 for s in sizes) and sum(sizes) == 2048
    with pytest.raises(ValueError):
        rounding.round_shards([0.5, 0.5], 10, 3)


def test_segment_ratios_sec_5_2():
    """Different ratios across the model (Sec. 5.2): a compute-only segment gets ratios proportional to speed, a
    communication-only one an even split; per-segment ratios are never slower than the best single B for the whole model
    (any shared B is feasible for every segment); one segment is the base case; brute force on a two-device grid."""
    speed = (3.0, 1.0)
    stages = [(6.0, 0, 0, 0), (2.0, 0, 0, 0), (0, 0, 0.1, 4.0), (1.0, 0, 0.2, 3.0)]
    B, t = lp.shard_ratios_segments(speed, stages, [0, 2, 3, 4])
    np.testing.assert_allclose(B[0], [0.75, 0.25], atol=1e-9)          # compute only: proportional to speed (CP)
    np.testing.assert_allclose(B[1], [0.5, 0.5], atol=1e-9)            # communication only: even (EV)
    assert 0.5 - 1e-9 <= B[2][0] <= 0.75 + 1e-9                        # mixed: between EV and CP
    assert t == pytest.approx(lp.iteration_time_segments(B, speed, stages, [0, 2, 3, 4]), rel=1e-12)
    Bs, ts = lp.shard_ratios(speed, stages)
    assert t <= ts + 1e-12 and t < ts - 1e-3                           # strictly better here: the segments want different ratios
    B1, t1 = lp.shard_ratios_segments(speed, stages, [0, 4])
    assert t1 == pytest.approx(ts, rel=1e-9)
    # brute force: every segment's optimum over a fine grid of B_0 (m = 2)
    grid = np.linspace(0, 1, 20001)
    for k, (a, b) in enumerate([(0, 2), (2, 3), (3, 4)]):
        best = min(lp.iteration_time([x, 1 - x], speed, stages[a:b]) for x in grid)
        assert lp.iteration_time(B[k], speed, stages[a:b]) <= best + 1e-9
    with pytest.raises(ValueError):
        lp.shard_ratios_segments(speed, stages, [0, 2, 2, 4])
