"""Seeded sweeps of shapes and flags (all within the documented limits): quantizers bit for bit against
the oracle, products against the FP64 product, on shapes no other test names."""
import numpy as np
import pytest
import torch

from test_gpu_parity import assert_same_bytes, check_product, dev, host, mixed_matrix, mx, random_packed  # noqa: F401

pytestmark = pytest.mark.gpu


def test_sweep_row_quantizer(mx, orc):
    rng = np.random.default_rng(101)
    for case in range(40):
        rows, cols = int(rng.integers(1, 300)), 32 * int(rng.integers(1, 40))
        pad = 8 * int(rng.integers(0, 4))
        dtype = ("f32", "bf16")[case % 2]
        rnd, mode = int(rng.integers(0, 2)), int(rng.integers(0, 2))
        seed, tid, base = int(rng.integers(0, 2 ** 63)), int(rng.integers(0, 2 ** 32)), 8 * int(rng.integers(0, 2 ** 40))
        x = mixed_matrix(rows, cols + pad, seed=200 + case, dtype=dtype)[:, :cols]      # ld = cols + pad
        want = orc.quantize(np.ascontiguousarray(x), round=rnd, scale_mode=mode, seed=seed, tensor_id=tid, index_base=base)
        src = dev(mixed_matrix(rows, cols + pad, seed=200 + case, dtype=dtype), dtype)[:, :cols]
        got = mx.mx_quantize(src, rnd, mode, seed=seed, tensor_id=tid, index_base=base)
        what = "case %d: %dx%d ld %d %s round %d mode %d" % (case, rows, cols, cols + pad, dtype, rnd, mode)
        assert_same_bytes(got[1], want[1], what + " scales")
        assert_same_bytes(got[0], want[0], what + " codes")


def test_sweep_transposed_quantizer(mx, orc):
    rng = np.random.default_rng(102)
    shapes = [(32 * int(rng.integers(1, 30)), 32 * int(rng.integers(1, 30))) for _ in range(28)]
    shapes += [(4096 + 32 * int(rng.integers(0, 64)), 4096 + 32 * int(rng.integers(0, 40))) for _ in range(3)]   # wide tiles + tail
    shapes += [(32 * int(rng.integers(600, 900)), 32 * int(rng.integers(20, 30))) for _ in range(3)]            # tall and narrow
    for case, (rows, cols) in enumerate(shapes):
        dtype = ("bf16", "f32")[case % 2]
        round_t, round_row, pre = int(rng.integers(0, 2)), int(rng.integers(0, 2)), int(rng.integers(0, 2))
        mode, want_row = int(rng.integers(0, 2)), bool(rng.integers(0, 4) > 0)
        seed, base = int(rng.integers(0, 2 ** 63)), 8 * int(rng.integers(0, 2 ** 36))
        pad = 8 * int(rng.integers(0, 3))
        full = mixed_matrix(rows, cols + pad, seed=300 + case, dtype=dtype)
        kw = dict(round_t=round_t, tensor_id_t=6, pre_quant=pre, want_row=want_row, round_row=round_row, tensor_id_row=1,
                  scale_mode=mode, seed=seed, index_base=base)
        want = orc.quantize_transposed(np.ascontiguousarray(full[:, :cols]), **kw)
        got = mx.mx_quantize_transposed(dev(full, dtype)[:, :cols], **kw)
        what = "case %d: %dx%d ld %d %s t %d row %d pre %d mode %d" % (case, rows, cols, cols + pad, dtype, round_t, round_row, pre, mode)
        for g, w, nm in zip(got, want, ("codes_t", "scales_t", "codes_row", "scales_row")):
            if w is None:
                assert g is None
            else:
                assert_same_bytes(g, w, what + " " + nm)


def test_sweep_products(mx, orc):
    rng = np.random.default_rng(103)
    for case in range(36):
        m, n = int(rng.integers(1, 700)), int(rng.integers(1, 700))
        k = 32 * int(rng.integers(1, 12)) if case % 3 == 0 else 128 * int(rng.integers(1, 24))
        ac, as_ = random_packed(m, k, 400 + case)
        bc, bs = random_packed(n, k, 500 + case)
        out = torch.float32 if case % 4 else torch.bfloat16
        if n % 4 == 0 and case % 2:
            bias = rng.standard_normal(n).astype(np.float32)
            got = mx.mx_linear_fwd_bias(dev(ac), dev(as_), dev(bc), dev(bs), dev(bias), out_dtype=torch.float32)
            ref = orc.gemm_f64(ac, as_, bc, bs) + bias.astype(np.float64)[None, :]
            absref = np.abs(orc.dequantize(ac, as_)) @ np.abs(orc.dequantize(bc, bs)).T + np.abs(bias)[None, :]
            err = np.abs(host(got).astype(np.float64) - ref)
            assert np.all(err <= 1e-5 * absref), ("case %d: %dx%dx%d with bias" % (case, m, n, k), (err / absref).max())
            continue
        got = mx.mx_linear_fwd(dev(ac), dev(as_), dev(bc), dev(bs), out_dtype=out).float()
        check_product(orc, got, ac, as_, bc, bs, "case %d: %dx%dx%d" % (case, m, n, k),
                      tol=1e-5 if out == torch.float32 else 2.0 ** -8)
