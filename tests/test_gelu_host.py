"""Host-side check of the fused stage's FP32 GELU: the constants in the HIP source, run through an FP32
emulation of the kernel's operation sequence, against the oracle's FP64 GELU (the tolerance stated at the
interface: 2^-18 |A| + 2^-120 for an exact pre-activation)."""
import os
import re

import numpy as np

from paper_2502_20853_amd import fit_gelu_erfcx as fg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _constants_in_source():
    src = open(os.path.join(ROOT, "paper_2502_20853_amd", "csrc", "mx_gemm.hip")).read()
    body = src[src.index("float gelu_f32(float x)"):]
    body = body[:body.index("\n}\n")]
    t0 = float(re.search(r"T0 = ([-0-9.e]+)f", body).group(1))
    coef = [float(re.search(r"C%d = ([-0-9.e]+)f" % i, body).group(1)) for i in range(9)]
    return coef, t0


def test_source_constants_are_the_fitted_ones():
    coef, t0 = _constants_in_source()
    fitted, ft0, err = fg.fit()
    assert err < 1e-7
    assert abs(t0 - ft0) < 1e-7
    np.testing.assert_allclose(coef, fitted, rtol=0, atol=2e-7)


def test_fp32_sequence_meets_the_stated_tolerance(orc):
    coef, t0 = _constants_in_source()
    rng = np.random.default_rng(5)
    xs = np.concatenate([np.linspace(-17.5, 17.5, 200001), rng.standard_normal(200000) * 3,
                         rng.uniform(-14, -4, 100000), np.array([0.0, -0.0, 1e-30, -1e-30, 100.0, -100.0, 3e38, -3e38])])
    xs = xs.astype(np.float32)
    got = fg.gelu_fp32(xs, coef, t0).astype(np.float64)
    want = orc.gelu(xs.astype(np.float64))
    tol = 2.0 ** -18 * np.abs(want) + 2.0 ** -120
    bad = np.abs(got - want) > tol
    assert not bad.any(), (xs[bad][:5], got[bad][:5], want[bad][:5])
    assert np.isfinite(got).all()
