"""GPU test of the entry point that allocates nothing: hap_sfb_grad_static keeps its split-K partial tiles in an array
of the library's device image and must return what hap_sfb_grad returns with a caller workspace - on two calls in a
row, the second with a smaller input (the array keeps the first call's contents), and after unrelated work."""
import numpy as np
import pytest

from hapgen import TensorId as T
from oracle import sfb as osfb

pytestmark = pytest.mark.gpu

from gpu_util import gen, empty, host, check, torch_mod  # noqa: E402


@pytest.fixture(scope="module")
def hap():
    import paper_2401_05965_amd as h
    return h


def _factors(seed, rows, in_f, out_f, dtype):
    Xh, Xd, Yh, Yd = [], [], [], []
    for i, r in enumerate(rows):
        a, b = gen(seed, T.SFB_X + i, (max(r, 1), in_f), 1.0, dtype); Xh.append(a); Xd.append(b)
        a, b = gen(seed, T.SFB_DY + i, (max(r, 1), out_f), 1.0, dtype); Yh.append(a); Yd.append(b)
    return Xh, Xd, Yh, Yd


def test_sfb_grad_static_matches_sfb_grad_on_two_calls_in_a_row(hap):
    torch = torch_mod()
    # (dtype, rows per device, in, out): a deep contraction over a small output (split over idle compute units, so the
    # scratch array is really used), then a smaller one, then fp32 at config 1's size
    cases = [("bf16", [1970, 1379, 788, 0, 591], 1024, 1536), ("bf16", [300, 77, 130], 264, 520), ("f32", [38, 26], 1024, 1024)]
    for dtype, rows, in_f, out_f in cases:
        io = hap.BF16 if dtype == "bf16" else hap.F32
        Xh, Xd, Yh, Yd = _factors(11, rows, in_f, out_f, dtype)
        ws = empty((hap.hap_sfb_workspace(len(rows), rows, in_f, out_f),), "u8")
        want = empty((in_f, out_f), "f32", float("nan")); got = empty((in_f, out_f), "f32", float("nan"))
        hap.hap_sfb_grad(Xd, Yd, rows, in_f, out_f, in_f, out_f, io, want, out_f, ws=ws)
        hap.hap_sfb_grad_static(Xd, Yd, rows, in_f, out_f, in_f, out_f, io, got, out_f)
        torch.cuda.synchronize()
        assert torch.equal(got, want), (dtype, rows)                       # same kernels, same split: bit-identical
        check(f"sfb static {dtype}", host(got), osfb.sfb_grad(Xh, Yh, rows), dtype)
        # accumulate = 1 on top of the first result
        hap.hap_sfb_grad(Xd, Yd, rows, in_f, out_f, in_f, out_f, io, want, out_f, accumulate=True, ws=ws)
        hap.hap_sfb_grad_static(Xd, Yd, rows, in_f, out_f, in_f, out_f, io, got, out_f, accumulate=True)
        torch.cuda.synchronize()
        assert torch.equal(got, want), (dtype, rows, "accumulate")


def test_sfb_grad_static_rejects_outputs_beyond_its_scratch(hap):
    t = empty((8, 8), "bf16", 0); dW = empty((8, 8), "f32", 0)
    with pytest.raises(hap.HapError) as e:
        hap.hap_sfb_grad_static([t], [t], [8], 4096, 16384, 4096, 16384, hap.BF16, dW, 16384)      # config 3's 64 Mi elements
    assert e.value.status == 7 and "scratch" in str(e.value)
