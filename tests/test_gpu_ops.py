"""Parity of single operations (RMSNorm, the three GEMM epilogues) against the CPU oracle, through
the C ABI, at shapes that span several tiles and ragged tails in M, N and K."""
import numpy as np
import pytest

from oracle import decoder as O
from tests import _util as U

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch


@pytest.mark.parametrize("fp32", [False, True], ids=["bf16", "fp32dbg"])
@pytest.mark.parametrize("T,H", [(1, 256), (7, 256), (130, 4096), (3, 8192), (5, 688)])
def test_rmsnorm(torch, fp32, T, H):
    from paper_2412_17246_amd import op_rmsnorm
    rng = np.random.default_rng([7, T, H])
    x, xr = U.f64_to_device(rng.standard_normal((T, H)) * 3.0, fp32)
    g, gr = U.f64_to_device(1.0 + 0.1 * rng.standard_normal(H), False)
    y = torch.empty_like(x)
    op_rmsnorm(x, g, y, 1e-5, fp32_debug=fp32)
    want = O.rmsnorm(xr, gr, 1e-5)
    err = U.rel_err(U.from_device(y), want)
    assert err <= (U.FP32_TOL if fp32 else U.BF16_TOL), err
    U.assert_rms(U.from_device(y), want, U.RMS_FP32 if fp32 else U.RMS_BF16_OP)


def test_rmsnorm_constant_vector(torch):
    from paper_2412_17246_amd import op_rmsnorm
    x = torch.full((2, 256), 3.0, dtype=torch.bfloat16, device="cuda")
    g = torch.ones(256, dtype=torch.bfloat16, device="cuda")
    y = torch.empty_like(x)
    op_rmsnorm(x, g, y, 1e-5)
    want = 3.0 / np.sqrt(9.0 + 1e-5)
    assert np.max(np.abs(U.from_device(y) - want)) <= 2 ** -8


GEMM_SHAPES = [
    # M, N, K: single tile, ragged M, ragged N (not a multiple of 32), K tail (688 = 10*64 + 48)
    (64, 128, 64), (1, 768, 256), (65, 768, 256), (200, 688, 256), (333, 256, 688), (130, 1376, 2048),
    (257, 4096, 512), (31, 48, 72),
    # large-tile kernel (M > 256, K a multiple of 64): ragged M, N tails, one and many K tiles
    (300, 768, 256), (700, 688, 1024), (513, 520, 64), (1030, 1024, 2048), (257, 132, 128),
    # more than 256 tiles with a small last round (272 / 544 tiles): with a workspace the last tiles are split over K
    (4300, 4092, 1024),
    # decode-sized problems (M <= 64, K a multiple of 64): the split-K kernel when a workspace is given
    (64, 4096, 4096), (33, 688, 1024), (7, 260, 640), (48, 1024, 14336),
    # 65..128 rows: the same kernel, two 64-row blocks per tile and k-slice (second block ragged)
    (128, 1024, 4096), (97, 688, 1024), (100, 256, 4096), (250, 512, 2048),
    # a few hundred rows, fewer tiles than CUs: every tile of the large-tile kernel split over K
    (200, 4096, 2048), (600, 1376, 4096),
    # decode-sized with a power-of-two row pitch and 32 k-tiles per workgroup: tiles start their walk over K at different places
    (40, 7168, 4096), (150, 7168, 4096),
]


@pytest.mark.parametrize("fp32", [False, True], ids=["bf16", "fp32dbg"])
@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm(torch, fp32, mode, M, N, K):
    from paper_2412_17246_amd import op_gemm
    rng = np.random.default_rng([11, mode, M, N, K])
    a, ar = U.f64_to_device(rng.standard_normal((M, K)), fp32)
    rows = 2 * N if mode == 2 else N
    w, wr = U.f64_to_device(rng.standard_normal((rows, K)) * (2.0 / np.sqrt(K)), False)
    r, rr = U.f64_to_device(rng.standard_normal((M, N)), fp32)
    c = torch.zeros_like(r)
    from paper_2412_17246_amd import op_gemm_workspace_bytes
    nws = op_gemm_workspace_bytes(mode, M, N, K, fp32_debug=fp32)
    ws = torch.empty(max(nws, 16), dtype=torch.uint8, device="cuda")
    op_gemm(mode, a, w, r if mode == 1 else None, c, M, N, K, fp32_debug=fp32, workspace=ws if nws else None)
    if nws and not fp32:
        # the same problem without a workspace takes the kernel that needs none; both must pass
        c2 = torch.zeros_like(r)
        op_gemm(mode, a, w, r if mode == 1 else None, c2, M, N, K)
    else:
        c2 = None
    if mode == 0:
        want = O.linear(ar, wr)
    elif mode == 1:
        want = rr + O.linear(ar, wr)
    else:
        want = O.swiglu(ar, wr[:N], wr[N:])
    got = U.from_device(c)
    err = U.rel_err(got, want)
    assert err <= (U.FP32_TOL if fp32 else U.BF16_TOL), err
    U.assert_rms(got, want, U.RMS_FP32 if fp32 else U.RMS_BF16_OP)
    if not fp32:
        # bf16 output rounding alone bounds the error far below the gate; a wrong tile would not
        assert U.mixed_err(got, want, 8e-3) <= 1.0
    if c2 is not None:
        assert U.rel_err(U.from_device(c2), want) <= U.BF16_TOL


@pytest.mark.parametrize("case", range(10))
def test_gemm_random_problems(torch, case):
    """Seeded random problems: any N (odd ones take the element-wise store path), K any multiple of 8, row counts on
    both sides of every kernel boundary; all three modes, both builds."""
    import random
    rnd = random.Random(case)
    M = rnd.choice([1, 2, 63, 64, 65, 255, 256, 257, rnd.randint(1, 900)])
    N = rnd.choice([rnd.randint(1, 1500), 4 * rnd.randint(1, 400), 8 * rnd.randint(1, 300), 256 * rnd.randint(1, 6)])
    K = 8 * rnd.choice([rnd.randint(1, 300), 8 * rnd.randint(1, 64)])
    for mode in (0, 1, 2):
        for fp32 in (False, True):
            test_gemm(torch, fp32, mode, M, N, K)


def test_gemm_residual_in_place_and_identity(torch):
    from paper_2412_17246_amd import op_gemm
    M, N = 150, 256
    rng = np.random.default_rng(5)
    a, ar = U.f64_to_device(rng.standard_normal((M, N)), False)
    eye = torch.eye(N, dtype=torch.bfloat16, device="cuda")
    x, xr = U.f64_to_device(rng.standard_normal((M, N)), False)
    op_gemm(1, a, eye, x, x, M, N, N)           # x <- x + a, residual aliased with the output
    got = U.from_device(x)
    want = U.f64(__import__("workloads").bf16_bits_from_f32((xr + ar).astype(np.float32)))
    assert np.array_equal(got, want)            # one rounding of an exact sum


@pytest.mark.parametrize("M,N,K", [(100, 512, 1024), (600, 1376, 4096), (4300, 4096, 1024)])
def test_gemm_residual_in_place_with_split_schedules(torch, M, N, K):
    # the residual aliased with the output, in the schedules that go through partial sums or partial tiles
    from paper_2412_17246_amd import op_gemm, op_gemm_workspace_bytes
    rng = np.random.default_rng([17, M, N, K])
    a, ar = U.f64_to_device(rng.standard_normal((M, K)), False)
    w, wr = U.f64_to_device(rng.standard_normal((N, K)) * (2.0 / np.sqrt(K)), False)
    x, xr = U.f64_to_device(rng.standard_normal((M, N)), False)
    nws = op_gemm_workspace_bytes(1, M, N, K)
    assert nws > 0
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    op_gemm(1, a, w, x, x, M, N, K, workspace=ws)
    assert U.rel_err(U.from_device(x), xr + O.linear(ar, wr)) <= U.BF16_TOL


def test_gemm_is_deterministic(torch):
    from paper_2412_17246_amd import op_gemm
    M, N, K = 300, 768, 688
    rng = np.random.default_rng(9)
    a, _ = U.f64_to_device(rng.standard_normal((M, K)), False)
    w, _ = U.f64_to_device(rng.standard_normal((N, K)) * 0.05, False)
    c1 = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    c2 = torch.empty_like(c1)
    op_gemm(0, a, w, None, c1, M, N, K)
    op_gemm(0, a, w, None, c2, M, N, K)
    torch.cuda.synchronize()
    assert torch.equal(c1.view(torch.int16), c2.view(torch.int16))
    # split last round: partial tiles are added in a fixed order
    from paper_2412_17246_amd import op_gemm_workspace_bytes
    M, N, K = 4352, 4096, 512
    nws = op_gemm_workspace_bytes(0, M, N, K)
    assert nws > 0
    a, _ = U.f64_to_device(rng.standard_normal((M, K)), False)
    w, _ = U.f64_to_device(rng.standard_normal((N, K)) * 0.05, False)
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    c1 = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    c2 = torch.empty_like(c1)
    op_gemm(0, a, w, None, c1, M, N, K, workspace=ws)
    ws.fill_(0xFF)                               # stale scratch contents must not matter
    op_gemm(0, a, w, None, c2, M, N, K, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(c1.view(torch.int16), c2.view(torch.int16))
