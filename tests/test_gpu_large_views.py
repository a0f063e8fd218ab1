"""Products whose operand views reach 2 GiB: the GEMM engine cuts them on the host into row blocks (K-contiguous
operand) or contraction segments (M- / N-contiguous operand), because its kernels address an operand with 32-bit
offsets.  The cutting is exercised twice: on ordinary sizes with the threshold lowered through the library's
testing aid (every element against the oracle, all four sharding modes), and once for real on a 2.25 GB activation
matrix (sampled rows / columns the oracle can compute one by one)."""
import numpy as np
import pytest

from oracle import linear as olin

pytestmark = pytest.mark.gpu

from gpu_util import check, host, torch_mod  # noqa: E402
from test_gpu_linear_sfb import run_linear_case  # noqa: E402


@pytest.fixture(scope="module")
def hap():
    import paper_2401_05965_amd as h
    return h


@pytest.mark.parametrize("dtype,limit", [("bf16", 600 << 10), ("f32", 1200 << 10), ("bf16", 64 << 10)])
@pytest.mark.parametrize("mode", [0, 1, 2, 3])
def test_cut_products_match_the_oracle_with_a_lowered_threshold(hap, dtype, limit, mode):
    """1500 x 776 x 520 with views cut at 600 KB: forward X is cut into row blocks and W into 2 contraction segments,
    bwd-data cuts dY by rows and W by columns of dX, bwd-weight becomes 4 segments.  At 64 KB the pieces would be too
    many (or too thin) and the product runs uncut: the result must not depend on the threshold."""
    offsets = {0: [0, 700, 700, 1500], 1: [0, 300, 520], 2: [0, 390, 776], 3: [0, 1]}[mode]
    try:
        before = hap.hap_debug_set_gemm_view_limit(limit)
        run_linear_case(hap, dtype, 1500, 776, 520, mode, offsets, act=(mode == 1), bias=True, full=True)
    finally:
        after = hap.hap_debug_set_gemm_view_limit(0)
    assert (after > before) == (limit > (64 << 10)), (before, after)


def test_activation_matrix_beyond_2_gib(hap):
    torch = torch_mod()
    M, K, N = 1_100_000, 1024, 256                      # X: 2.25 GB of bf16
    g = torch.Generator(device="cuda"); g.manual_seed(11)
    X = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    for lo in range(0, M, 100_000):                     # filled in slabs: the fp32 temporary stays small
        X[lo:lo + 100_000] = torch.randn((min(100_000, M - lo), K), generator=g, device="cuda").to(torch.bfloat16)
    W = (torch.randn((K, N), generator=g, device="cuda") * 0.05).to(torch.bfloat16)
    b = (torch.randn((N,), generator=g, device="cuda") * 0.5).to(torch.bfloat16)
    dY = torch.randn((M, N), generator=g, device="cuda").to(torch.bfloat16)
    assert X.numel() * 2 > 2**31
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    dX = torch.zeros((M, K), dtype=torch.bfloat16, device="cuda")
    dW = torch.zeros((K, N), dtype=torch.float32, device="cuda")
    db = torch.zeros((N,), dtype=torch.float32, device="cuda")
    d = hap.LinearDesc(M, K, N, hap.REPLICATED, [0, 1], hap.BF16, has_bias=True, ldx=K, ldw=N, ldy=N)
    ws = torch.empty((hap.hap_linear_bwd_workspace(d, 0),), dtype=torch.uint8, device="cuda")
    before = hap.hap_debug_set_gemm_view_limit(0)
    hap.hap_sharded_linear_fwd(d, 0, X, W, b, Y, None, ws)
    hap.hap_sharded_linear_bwd(d, 0, X, W, None, dY, dX, dW, hap.F32, db, ws)
    assert hap.hap_debug_set_gemm_view_limit(0) - before == 2      # forward (row blocks of X) and bwd-weight (segments); dX has small operands
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([[0, 255, 256, M - 1, M - 257], rng.integers(0, M, 40),
                                     np.arange(1, 5) * (M // 5) + rng.integers(-300, 300, 4)]))
    ridx = torch.from_numpy(rows).cuda()
    Wh, bh = host(W), host(b)
    Xr, dYr = host(X[ridx]), host(dY[ridx])
    Yo, _ = olin.linear_fwd(Xr, Wh, bh, False)
    check("Y rows", host(Y[ridx]), Yo, "bf16")
    check("dX rows", host(dX[ridx]), dYr @ Wh.T, "bf16")
    # weight-gradient rows (= columns of X) are independent of each other: a sample of them is an exact sub-problem
    cols = np.unique(np.concatenate([[0, 255, 256, K - 1], rng.integers(0, K, 4)]))
    dYh = host(dY)
    Xc = host(X[:, torch.from_numpy(cols).cuda()])
    check("dW rows", host(dW)[cols], Xc.T @ dYh, "bf16")
    check("db", host(db), dYh.sum(0), "bf16")
