"""bz_op_gemm_static - the GEMM entry point that allocates nothing - through the C ABI, against
bz_op_gemm with a caller's workspace: same kernels and schedules, so the outputs must be the same bits.
Two calls in a row share the library's static scratch, the second with a smaller input, and each is
also held to the oracle.  Collected last on purpose."""
import numpy as np
import pytest

from oracle import decoder as O
from tests import _util as U


@pytest.mark.gpu
@pytest.mark.parametrize("fp32", [False, True], ids=["bf16", "fp32dbg"])
@pytest.mark.parametrize("mode,first,second", [
    # split-K partial sums (decode-sized): 64 rows, then 33 rows of a narrower matrix
    (1, (64, 4096, 4096), (33, 688, 1024)),
    # partial tiles of the large-tile kernel's split last round, then a few hundred rows with every tile split
    (0, (4300, 4092, 1024), (600, 1376, 4096)),
    # SwiGLU epilogue behind split-K partial sums (two 64-row blocks), then a schedule that needs no scratch at all
    (2, (128, 1024, 4096), (31, 48, 72)),
])
def test_static_scratch_gemm_equals_workspace_gemm_on_two_calls_in_a_row(fp32, mode, first, second):
    import torch
    from paper_2412_17246_amd import op_gemm, op_gemm_static, op_gemm_workspace_bytes
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    cases = []
    for (M, N, K) in (first, second):
        rng = np.random.default_rng([23, mode, M, N, K])
        a, ar = U.f64_to_device(rng.standard_normal((M, K)), fp32)
        rows = 2 * N if mode == 2 else N
        w, wr = U.f64_to_device(rng.standard_normal((rows, K)) * (2.0 / np.sqrt(K)), False)
        r, rr = U.f64_to_device(rng.standard_normal((M, N)), fp32)
        nws = op_gemm_workspace_bytes(mode, M, N, K, fp32_debug=fp32)
        ws = torch.empty(max(nws, 16), dtype=torch.uint8, device="cuda")
        want_dev = torch.zeros_like(r)
        op_gemm(mode, a, w, r if mode == 1 else None, want_dev, M, N, K, fp32_debug=fp32, workspace=ws if nws else None)
        cases.append((M, N, K, a, ar, w, wr, r, rr, want_dev, torch.zeros_like(r)))
    torch.cuda.synchronize()
    # the two calls back to back on one stream, nothing between them: the second starts on the scratch the
    # first one left behind
    for (M, N, K, a, ar, w, wr, r, rr, want_dev, got_dev) in cases:
        op_gemm_static(mode, a, w, r if mode == 1 else None, got_dev, M, N, K, fp32_debug=fp32)
    torch.cuda.synchronize()
    for (M, N, K, a, ar, w, wr, r, rr, want_dev, got_dev) in cases:
        assert torch.equal(got_dev.view(torch.int32 if fp32 else torch.int16),
                           want_dev.view(torch.int32 if fp32 else torch.int16)), (M, N, K)
        if mode == 0:
            want = O.linear(ar, wr)
        elif mode == 1:
            want = rr + O.linear(ar, wr)
        else:
            want = O.swiglu(ar, wr[:N], wr[N:])
        assert U.rel_err(U.from_device(got_dev), want) <= (U.FP32_TOL if fp32 else U.BF16_TOL)


@pytest.mark.gpu
def test_static_scratch_gemm_after_the_scratch_was_overwritten():
    """Stale contents of the static scratch never reach a result: a large split problem fills it, then a
    smaller one whose partial tiles cover only its first part must still match the workspace call."""
    import torch
    from paper_2412_17246_amd import op_gemm, op_gemm_static, op_gemm_workspace_bytes
    rng = np.random.default_rng(29)
    outs = []
    for (M, N, K) in ((2000, 4096, 4096), (300, 768, 256)):
        a, _ = U.f64_to_device(rng.standard_normal((M, K)) * 50.0, False)
        w, _ = U.f64_to_device(rng.standard_normal((N, K)), False)
        x, _ = U.f64_to_device(rng.standard_normal((M, N)), False)
        nws = op_gemm_workspace_bytes(1, M, N, K)
        ws = torch.empty(max(nws, 16), dtype=torch.uint8, device="cuda")
        want = x.clone()
        op_gemm(1, a, w, want, want, M, N, K, workspace=ws if nws else None)
        outs.append((M, N, K, a, w, x, want))
    for (M, N, K, a, w, x, want) in outs:
        op_gemm_static(1, a, w, x, x, M, N, K)           # residual aliased with the output, as in a layer
    torch.cuda.synchronize()
    for (M, N, K, a, w, x, want) in outs:
        assert torch.equal(x.view(torch.int16), want.view(torch.int16)), (M, N, K)


def test_static_scratch_gemm_rejects_oversized_problems_before_touching_the_gpu():
    """No GPU needed: a problem whose partial sums exceed the static scratch is refused with BZ_ECAPACITY
    ahead of any HIP call (device pointers are never dereferenced on the host)."""
    from paper_2412_17246_amd import load_library, op_gemm_workspace_bytes
    from paper_2412_17246_amd.binding import BZ_STATIC_SCRATCH_BYTES
    lib = load_library(False)
    assert op_gemm_workspace_bytes(0, 256, 131072, 4096) > BZ_STATIC_SCRATCH_BYTES
    assert lib.bz_op_gemm_static(0, 1, 1, None, 1, 256, 131072, 4096, None) == -7       # BZ_ECAPACITY
    assert lib.bz_op_gemm_static(0, None, 1, None, 1, 64, 128, 64, None) == -1          # BZ_EINVAL: null operand
    assert lib.bz_op_gemm_static(1, 1, 1, None, 1, 64, 128, 64, None) == -1             # residual mode without a residual
