"""GPU test of mx_linear_bwd_dw_noalloc: the entry point for callers that cannot allocate.  Its K-split
partials live in a device array inside the library; the result must equal mx_linear_bwd_dw's (same
kernels, same summation order: bit for bit) and the FP64 oracle's to the products' tolerance, on two
calls in a row, the second with a smaller input that reuses the array the first one filled."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mx():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2502_20853_amd import binding
    binding.lib()
    return binding


def _random_packed(rows, k, seed):
    rng = np.random.default_rng(seed)
    codes = rng.integers(0, 256, (rows, k // 2), dtype=np.uint8)
    scales = rng.integers(118, 132, (rows, k // 32), dtype=np.uint8)
    return codes, scales


def test_no_alloc_dw_equals_the_workspace_entry_point_twice(mx, orc):
    # (C, D, N): a K-split product over several 256 x 256 tiles, then a smaller one whose partials
    # occupy the front of the array that still holds the first call's
    last_need = None
    for (C, D, N, seed) in ((768, 512, 16384, 1), (320, 264, 8192 + 128, 2)):
        a, a_s = _random_packed(C, N, seed)
        b, b_s = _random_packed(D, N, seed + 100)
        ad, asd, bd, bsd = (torch.from_numpy(t).cuda() for t in (a, a_s, b, b_s))
        need = mx.mx_linear_workspace_bytes(mx.GEMM_BWD_DW, N, C, D)
        assert 0 < need <= mx.NOALLOC_MAX_WORKSPACE_BYTES, "the case must take the K-split path"
        assert last_need is None or need < last_need
        last_need = need
        want = mx.mx_linear_bwd_dw(ad, asd, bd, bsd, out_dtype=torch.float32)
        got = torch.full((C, D), float("nan"), device="cuda")
        mx.mx_linear_bwd_dw_noalloc(ad, asd, bd, bsd, out=got)
        torch.cuda.synchronize()
        assert torch.equal(got, want), (C, D, N)
        ref = orc.gemm_f64(a, a_s, b, b_s)
        g = got.cpu().numpy().astype(np.float64)
        assert np.linalg.norm(g - ref) <= 1e-5 * np.linalg.norm(ref)
        absref = np.abs(orc.dequantize(a, a_s)).astype(np.float64) @ np.abs(orc.dequantize(b, b_s)).astype(np.float64).T
        assert np.all(np.abs(g - ref) <= 1e-5 * absref)
        # bf16 output through the same path
        want16 = mx.mx_linear_bwd_dw(ad, asd, bd, bsd, out_dtype=torch.bfloat16)
        got16 = torch.zeros((C, D), dtype=torch.bfloat16, device="cuda")
        mx.mx_linear_bwd_dw_noalloc(ad, asd, bd, bsd, out=got16)
        assert torch.equal(got16, want16)
