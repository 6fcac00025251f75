"""GPU tests at sizes whose element indices, byte offsets and counters leave 32 bits: sources of more
than 2^33 elements, packed outputs of more than 4 GiB, a product output of more than 4 GiB, and the
largest contraction length the products accept (2^24, operands of more than 4 GiB).  The oracle
checks row blocks placed on those boundaries (its counters continue through index_base) and sampled
product entries."""
import numpy as np
import pytest
import torch

from test_gpu_parity import assert_same_bytes, host, mixed_matrix, mx  # noqa: F401  (mx: the fixture)

pytestmark = pytest.mark.gpu


def _fill_normal(t, seed):
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    step = 1 << 16
    for r in range(0, t.shape[0], step):
        t[r:r + step].normal_(generator=gen)


def test_quantizers_beyond_32_bit_indices(mx, orc):
    """bf16 source [2^21 + 288, 4096]: 2^33 + ... elements (17 GB), packed outputs of 4.3 GB each.  Row
    blocks at element indices 0, 2^31, 2^32, 2^33 and the ragged end are overwritten with known data
    and compared bit for bit, for both fused passes of the layer and for the row quantizer alone
    (contiguous, and strided over the left half)."""
    rows, cols = (1 << 21) + 288, 4096
    seed, base = 0x1234567887654321, 1 << 36                      # counters with a non-zero high word
    X = torch.empty((rows, cols), dtype=torch.bfloat16, device="cuda")
    _fill_normal(X, 1)
    blocks = [(0, 512), ((1 << 19) - 256, (1 << 19) + 256), ((1 << 20) - 256, (1 << 20) + 256), ((1 << 21) - 256, rows)]
    known = []
    for i, (r0, r1) in enumerate(blocks):
        x = mixed_matrix(r1 - r0, cols, seed=40 + i, dtype="bf16")
        X[r0:r1] = torch.from_numpy(x).cuda().to(torch.bfloat16)
        known.append(x)
    out = None
    for name, kw in (("dY-type", dict(round_t=1, tensor_id_t=5, pre_quant=0, round_row=1, tensor_id_row=3)),
                     ("X-type", dict(round_t=1, tensor_id_t=6, pre_quant=1, round_row=0, tensor_id_row=1))):
        out = mx.mx_quantize_transposed(X, seed=seed, index_base=base, out=out, **kw)
        for (r0, r1), x in zip(blocks, known):
            want = orc.quantize_transposed(x, seed=seed, index_base=base + r0 * cols, **kw)
            what = "%s rows %d..%d " % (name, r0, r1)
            assert_same_bytes(out[3][r0:r1], want[3], what + "row scales")
            assert_same_bytes(out[2][r0:r1], want[2], what + "row codes")
            assert_same_bytes(out[1][:, r0 // 32:r1 // 32].contiguous(), want[1], what + "transposed scales")
            assert_same_bytes(out[0][:, r0 // 2:r1 // 2].contiguous(), want[0], what + "transposed codes")
    rows_out = (out[2], out[3])
    del out
    for name, src, c in (("contiguous", X, cols), ("strided", X[:, :cols // 2], cols // 2)):
        got = mx.mx_quantize(src, round=1, seed=seed, tensor_id=3, index_base=base,
                             out=(rows_out[0].view(-1)[: rows * c // 2].view(rows, c // 2),
                                  rows_out[1].view(-1)[: rows * c // 32].view(rows, c // 32)))
        for (r0, r1), x in zip(blocks, known):
            want = orc.quantize(x[:, :c], round=1, seed=seed, tensor_id=3, index_base=base + r0 * c)
            assert_same_bytes(got[1][r0:r1], want[1], "%s rows %d..%d scales" % (name, r0, r1))
            assert_same_bytes(got[0][r0:r1], want[0], "%s rows %d..%d codes" % (name, r0, r1))


def _random_operand(rng, rows, k):
    raw = np.random.PCG64(int(rng.integers(1 << 30))).random_raw(rows * (k // 2) // 8)   # 64 random bits per draw
    codes = raw.view(np.uint8).reshape(rows, k // 2)
    scales = rng.integers(122, 132, (rows, k // 32), dtype=np.uint8)
    return codes, scales


def _check_samples(orc, out, ops, ii, jj, bf16, what):
    ref, absref = orc.gemm_f64_sampled(*ops, ii, jj)
    got = host(out[torch.from_numpy(ii).cuda(), torch.from_numpy(jj).cuda()].float()).astype(np.float64)
    tol = 1e-5 * absref + (np.abs(ref) * 2.0 ** -8 if bf16 else 0.0)
    assert np.all(np.abs(got - ref) <= tol), (what, np.max(np.abs(got - ref) / (absref + 1e-300)))


@pytest.mark.parametrize("out_dtype", [torch.bfloat16, torch.float32])
def test_product_output_beyond_4GiB(mx, orc, out_dtype):
    """Y[2^20 + 785, 2304] (4.8 GB as bf16, 9.7 GB as FP32) from random packed operands, K = 512:
    sampled entries, the corners and entries beyond the 4 GiB offset among them."""
    N, C, D = (1 << 20) + 785, 2304, 512
    rng = np.random.default_rng(3)
    xq, xs = _random_operand(rng, N, D)
    wq, ws = _random_operand(rng, C, D)
    y = mx.mx_linear_fwd(*(torch.from_numpy(a).cuda() for a in (xq, xs, wq, ws)), out_dtype=out_dtype)
    torch.cuda.synchronize()
    ii = rng.integers(0, N, 512)
    jj = rng.integers(0, C, 512)
    ii[:4], jj[:4] = [0, N - 1, 0, N - 1], [0, 0, C - 1, C - 1]
    ii[4:132] = rng.integers(N - 1024, N, 128)                     # the last tiles, far beyond 4 GiB
    _check_samples(orc, y, (xq, xs, wq, ws), ii, jj, out_dtype == torch.bfloat16, "Y")


def test_weight_gradient_at_the_largest_contraction_length(mx, orc):
    """dW[544, 128] over N = 2^24 tokens, the largest contraction length accepted: operand rows of
    8 MiB, 4.6 GB of codes for dY^T (offsets beyond 4 GiB), K split over all compute units."""
    C, D, N = 544, 128, 1 << 24
    rng = np.random.default_rng(4)
    dytq, dyts = _random_operand(rng, C, N)
    xtq, xts = _random_operand(rng, D, N)
    dw = mx.mx_linear_bwd_dw(*(torch.from_numpy(a).cuda() for a in (dytq, dyts, xtq, xts)))
    torch.cuda.synchronize()
    ii = rng.integers(0, C, 48)
    jj = rng.integers(0, D, 48)
    ii[:4], jj[:4] = [0, C - 1, 0, C - 1], [0, 0, D - 1, D - 1]
    ii[4:12] = rng.integers(513, C, 8)                             # rows whose codes start beyond 4 GiB
    _check_samples(orc, dw, (dytq, dyts, xtq, xts), ii, jj, False, "dW")
