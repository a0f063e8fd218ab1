"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its host
functions (LP, cost model, rounding, argument validation) agree with the oracle."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import lp as olp, rounding as ornd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def hap():
    import paper_2401_05965_amd as h
    return h


def test_every_declared_symbol_is_exported(hap):
    with open(os.path.join(ROOT, "include", "libhap.h")) as f:
        text = f.read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(hap_[a-z0-9_]+)\s*\(", text))
    assert len(names) >= 20
    for n in sorted(names):
        assert hasattr(hap.lib, n), f"{n} declared in libhap.h but not exported"
        assert callable(getattr(hap, n, None)), f"{n} has no Python binding of the same name"
    assert hap.lib.hap_version().startswith(b"libhap") and hap.hap_version().startswith("libhap")
    assert hap.hap_strerror(0) and hap.hap_last_error() is not None


def test_lp_matches_oracle_on_random_problems(hap):
    rng = np.random.default_rng(3)
    for trial in range(40):
        m = int(rng.integers(1, 9)); S = int(rng.integers(1, 6))
        speed = rng.uniform(0.2, 3.0, m)
        stages = [tuple(rng.uniform(0, 2, 4) * rng.integers(0, 2, 4)) for _ in range(S)]
        B, t = hap.hap_shard_ratios(speed, stages)
        Bo, to = olp.shard_ratios(speed, stages)
        assert abs(sum(B) - 1) < 1e-12 and min(B) >= 0
        assert t == pytest.approx(to, rel=1e-9, abs=1e-12)          # optimum value is unique, the argmin need not be
        assert hap.hap_iteration_time(speed, stages, B) == pytest.approx(olp.iteration_time(B, speed, stages), rel=1e-14)
        assert t == pytest.approx(olp.iteration_time(B, speed, stages), rel=1e-12)


def test_lp_compute_only_and_comm_only_closed_forms(hap):
    for speed in [(1.0, 0.67), (1.0, 0.6, 0.35), (1, 1, .5, .5), (1, .8, .8, .4, .25), tuple([1.0] * 8)]:
        B, _ = hap.hap_shard_ratios(speed, [(3.0e12, 0, 0, 0)])
        s = np.asarray(speed, float)
        assert np.allclose(B, s / s.sum(), atol=1e-12)
        B, _ = hap.hap_shard_ratios(speed, [(0, 0, 1e-4, 0.5)])
        assert np.allclose(B, 1.0 / len(speed), atol=1e-12)
    # realistic magnitudes: flops ~1e12, speeds ~1e14 flops/s, seconds ~1e-3
    B, t = hap.hap_shard_ratios([1.2e14, 0.5e14], [(3.4e12, 1e10, 2e-5, 1.5e-3), (1.1e12, 0, 1e-5, 4e-4)])
    Bo, to = olp.shard_ratios([1.2e14, 0.5e14], [(3.4e12, 1e10, 2e-5, 1.5e-3), (1.1e12, 0, 1e-5, 4e-4)])
    assert t == pytest.approx(to, rel=1e-9)


def test_lp_solves_in_under_a_millisecond(hap):
    import time
    speed = [1, .8, .8, .4, .25]; stages = [(5.0, 0.5, 1e-3, 1.0)] * 4 + [(2.0, 0.0, 1e-3, 0.3)] * 4
    hap.hap_shard_ratios(speed, stages)
    t0 = time.perf_counter()
    for _ in range(100):
        hap.hap_shard_ratios(speed, stages)
    assert (time.perf_counter() - t0) / 100 < 1e-3       # the paper reports < 1 ms for its solver (Sec. 7.8)


def test_rounding_bit_exact_vs_oracle(hap):
    rng = np.random.default_rng(9)
    for trial in range(300):
        m = int(rng.integers(1, 9))
        r = rng.dirichlet(np.ones(m) * rng.uniform(0.2, 3))
        g = int(rng.choice([1, 1, 1, 2, 8, 128]))
        n = int(rng.integers(0, 5000)) * g
        assert hap.hap_round_shards(r, n, g) == ornd.round_shards(r, n, g)
    for speeds, n, g, want in [((1, .8, .8, .4, .25), 256, 1, [79, 63, 63, 31, 20]), ((1, .8, .8, .4, .25), 4096, 1, [1261, 1008, 1008, 504, 315]),
                               ((1, .6, .35), 16384, 1, [8402, 5041, 2941]), ((1, 1, .5, .5), 2048, 128, [640, 640, 384, 384]),
                               ((1, 1, .5, .5), 8192, 1, [2731, 2731, 1365, 1365]), ((1, .67), 64, 1, [38, 26])]:
        B, _ = hap.hap_shard_ratios(speeds, [(1.0, 0, 0, 0)])
        sizes, offs = hap.hap_round_shards(B, n, g)
        assert sizes == want and offs[-1] == n


def test_host_side_argument_errors(hap):
    E = hap.HapError
    with pytest.raises(E) as e:
        hap.hap_shard_ratios([1.0, -1.0], [(1, 0, 0, 0)])
    assert e.value.status == 1
    with pytest.raises(E) as e:
        hap.hap_shard_ratios([1.0], [(1, 0, 0, -2.0)])
    assert e.value.status == 1
    with pytest.raises(E) as e:
        hap.hap_round_shards([0.5, 0.5], 10, 3)
    assert e.value.status == 2
    with pytest.raises(E) as e:
        hap.hap_round_shards([0.9, 0.5], 10, 1)
    assert e.value.status == 1
    # device entry points validate on the host before any launch: these fail without touching a GPU
    z = C.c_void_p(0)
    d = hap.LinearDesc(8, 8, 8, hap.SHARD_FEATURE, [0, 4, 9], hap.BF16)
    assert hap.lib.hap_sharded_linear_fwd(C.byref(d.c), 0, z, z, z, z, z, z, C.c_size_t(0), z) == 2   # offsets do not end at the dimension
    d = hap.LinearDesc(8, 8, 8, hap.SHARD_FEATURE, [0, 5, 3, 8], hap.BF16)
    assert hap.lib.hap_sharded_linear_fwd(C.byref(d.c), 0, z, z, z, z, z, z, C.c_size_t(0), z) == 2   # not monotone
    d = hap.LinearDesc(8, 8, 8, hap.SHARD_FEATURE, [0, 4, 8], hap.BF16)
    assert hap.lib.hap_sharded_linear_fwd(C.byref(d.c), 2, z, z, z, z, z, z, C.c_size_t(0), z) == 1   # shard index out of range
    assert hap.lib.hap_sharded_linear_fwd(C.byref(d.c), 0, z, z, z, z, z, z, C.c_size_t(0), z) == 1   # NULL tensors
    assert b"NULL" in hap.lib.hap_last_error()
    d = hap.LinearDesc(8, 8, 8, hap.SHARD_REDUCTION, [0, 4, 8], hap.BF16, has_bias=True)
    assert hap.lib.hap_sharded_linear_fwd(C.byref(d.c), 0, z, z, z, z, z, z, C.c_size_t(0), z) == 1   # bias on a partial
    d = hap.LinearDesc(8, 8, 8, hap.SHARD_FEATURE, [0, 4, 8], hap.BF16, ldw=4)
    assert hap.lib.hap_sharded_linear_fwd(C.byref(d.c), 0, z, z, z, z, z, z, C.c_size_t(0), z) == 2   # ld below width
    d = hap.LinearDesc(8, 8, 8, hap.SHARD_FEATURE, [0, 0, 8], hap.BF16)
    assert hap.lib.hap_sharded_linear_fwd(C.byref(d.c), 0, z, z, z, z, z, z, C.c_size_t(0), z) == 0   # empty shard: OK, no launch
    rows = (C.c_int64 * 1)(-1)
    ptrs = (C.c_void_p * 1)(0)
    one = C.c_void_p(16)
    assert hap.lib.hap_sfb_grad(1, ptrs, ptrs, rows, C.c_int64(8), C.c_int64(8), C.c_int64(8), C.c_int64(8), 1, one, C.c_int64(8), 0, z, C.c_size_t(0), z) == 1
    assert hap.lib.hap_sfb_grad(65, ptrs, ptrs, rows, C.c_int64(8), C.c_int64(8), C.c_int64(8), C.c_int64(8), 1, one, C.c_int64(8), 0, z, C.c_size_t(0), z) == 1
    assert hap.lib.hap_strerror(5) == b"workspace missing or too small"


def test_moe_host_side_argument_errors(hap):
    """Expert-sharded layer (Sec. 7.6): descriptor and pointer checks happen before any launch."""
    z = C.c_void_p(0)
    fwd = lambda d, j: hap.lib.hap_moe_linear_fwd(C.byref(d.c), j, z, z, z, z, z, z, z, C.c_size_t(0), z)
    d = hap.MoeDesc(7, 16, 8, 8, [0, 3, 5, 6, 8], hap.BF16)
    assert fwd(d, 0) == 2                                                   # expert ranges do not end at the expert count
    d = hap.MoeDesc(7, 16, 8, 8, [0, 3, 5, 6, 7], hap.BF16)
    assert fwd(d, 4) == 1                                                   # device index out of range
    assert fwd(d, 1) == 1 and b"NULL" in hap.lib.hap_last_error()           # NULL tensors
    d = hap.MoeDesc(7, 16, 8, 8, [0, 3, 5, 7, 7], hap.BF16)
    assert fwd(d, 3) == 0                                                   # a device without experts: OK, no launch
    assert hap.hap_moe_linear_bwd_workspace(d, 3) == 0
    d = hap.MoeDesc(7, 16, 8, 8, [0, 3, 5, 6, 7], hap.BF16, ldy=4)
    assert fwd(d, 0) == 2                                                   # ld below width
    d = hap.MoeDesc(7, 16, 8, 8, [0, 3, 5, 6, 7], hap.BF16, act=hap.ACT_GELU_ERF, has_bias=True)
    one = C.c_void_p(256)
    assert hap.lib.hap_moe_linear_fwd(C.byref(d.c), 0, one, one, z, z, one, z, z, C.c_size_t(0), z) == 1            # has_bias without a bias pointer
    need = hap.hap_moe_linear_bwd_workspace(d, 0)
    assert need >= 3 * 16 * 8 * 2
    assert hap.lib.hap_moe_linear_bwd(C.byref(d.c), 0, one, one, one, one, z, one, one, 1, z, z, C.c_size_t(0), z) == 5   # workspace missing
    assert hap.lib.hap_moe_linear_bwd(C.byref(d.c), 0, one, one, z, one, z, one, one, 1, z, one, C.c_size_t(need), z) == 1  # no saved pre-activation
    assert hap.lib.hap_moe_linear_bwd(C.byref(d.c), 0, one, one, one, one, z, one, one, 7, z, one, C.c_size_t(need), z) == 1  # bad dW dtype


def test_allgather_host_side_argument_errors(hap):
    """Uneven All-Gather data movement (Sec. 2.3.1): descriptor checks and the padded-slot capacity need no GPU."""
    z = C.c_void_p(0)
    d = hap.GatherDesc(100, 64, 0, [0, 50, 81, 100], 2)
    assert hap.hap_allgather_capacity(d) == 50
    d1 = hap.GatherDesc(64, 100, 1, [0, 10, 10, 100], 4)
    assert hap.hap_allgather_capacity(d1) == 90
    assert hap.hap_allgather_capacity(hap.GatherDesc(100, 64, 0, [0, 50, 99], 2)) == -1          # ranges do not end at the axis length
    assert hap.hap_allgather_capacity(hap.GatherDesc(100, 64, 2, [0, 50, 100], 2)) == -1         # bad dim
    assert hap.hap_allgather_capacity(hap.GatherDesc(100, 64, 0, [0, 50, 100], 3)) == -1         # bad element size
    assert hap.lib.hap_allgather_pad(C.byref(d.c), 3, z, C.c_int64(64), z, C.c_int64(64), z) == 1   # device index out of range
    assert hap.lib.hap_allgather_pad(C.byref(d.c), 0, z, C.c_int64(64), z, C.c_int64(64), z) == 1   # NULL pointers
    one = C.c_void_p(256)
    assert hap.lib.hap_allgather_pad(C.byref(d.c), 0, one, C.c_int64(63), one, C.c_int64(64), z) == 2   # ld below width
    assert hap.lib.hap_allgather_pad(C.byref(d1.c), 1, z, C.c_int64(0), z, C.c_int64(0), z) == 0        # empty shard: OK, no launch
    ptrs = (C.c_void_p * 3)(256, 0, 256)
    lds = (C.c_int64 * 3)(10, 0, 89)
    assert hap.lib.hap_allgather_assemble(C.byref(d1.c), ptrs, lds, one, C.c_int64(100), z) == 2    # piece 2: ld 89 < its 90 columns
    assert hap.lib.hap_allgather_assemble(C.byref(d1.c), ptrs, lds, one, C.c_int64(99), z) == 2     # ld_out below cols
    assert hap.lib.hap_allgather_assemble(C.byref(d1.c), z, lds, one, C.c_int64(100), z) == 1
    # the reverse movement before a padded Reduce-Scatter: slots of capacity 90 columns each
    slots = (C.c_void_p * 3)(256, 256, 256)
    assert hap.lib.hap_reducescatter_split(C.byref(d1.c), one, C.c_int64(99), slots, (C.c_int64 * 3)(90, 90, 90), z) == 2    # ld_full below cols
    assert hap.lib.hap_reducescatter_split(C.byref(d1.c), one, C.c_int64(100), slots, (C.c_int64 * 3)(90, 89, 90), z) == 2   # slot 1 narrower than the capacity
    assert hap.lib.hap_reducescatter_split(C.byref(d1.c), z, C.c_int64(100), slots, (C.c_int64 * 3)(90, 90, 90), z) == 1     # full is NULL
    assert hap.lib.hap_reducescatter_split(C.byref(d1.c), one, C.c_int64(100), (C.c_void_p * 3)(256, 0, 256), (C.c_int64 * 3)(90, 90, 90), z) == 1   # the empty shard still has a slot
    assert hap.lib.hap_reducescatter_split(C.byref(d1.c), one, C.c_int64(100), z, z, z) == 1


def test_segment_ratios_match_oracle(hap):
    """Per-segment ratios (Sec. 5.2): objective parity with the oracle on random staged models, ratios where unique."""
    from oracle import lp as olp
    rng = np.random.default_rng(5)
    for trial in range(20):
        m = int(rng.integers(2, 6)); n = int(rng.integers(2, 9))
        speed = rng.uniform(0.2, 2.0, m)
        stages = [(float(rng.uniform(0, 5)), float(rng.uniform(0, 1)), float(rng.uniform(0, 0.2)), float(rng.uniform(0, 4))) for _ in range(n)]
        cuts = sorted(set([0, n] + [int(c) for c in rng.integers(1, n, size=int(rng.integers(0, 3)))]))
        Bo, to = olp.shard_ratios_segments(speed, stages, cuts)
        B, t = hap.hap_shard_ratios_segments(speed, stages, cuts)
        assert t == pytest.approx(to, rel=1e-9, abs=1e-12)
        assert hap.hap_iteration_time_segments(speed, stages, cuts, B) == pytest.approx(t, rel=1e-12)
        assert all(abs(sum(row) - 1) < 1e-12 and min(row) >= 0 for row in B)
    B, t = hap.hap_shard_ratios_segments((3.0, 1.0), [(6.0, 0, 0, 0), (0, 0, 0.1, 4.0)], [0, 1, 2])
    assert B[0] == pytest.approx([0.75, 0.25], abs=1e-12) and B[1] == pytest.approx([0.5, 0.5], abs=1e-12)
    with pytest.raises(hap.HapError) as e:
        hap.hap_shard_ratios_segments((1.0, 1.0), [(1, 0, 0, 0), (1, 0, 0, 0)], [0, 0, 2])
    assert e.value.status == 2
    with pytest.raises(hap.HapError) as e:
        hap.hap_shard_ratios_segments((1.0, 1.0), [(1, 0, 0, 0), (1, 0, 0, 0)], [0, 1])
    assert e.value.status == 2
