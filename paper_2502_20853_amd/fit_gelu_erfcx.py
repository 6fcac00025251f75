"""Coefficients of the FP32 GELU in the fused output stage (csrc/mx_gemm.hip, gelu_f32), and a check of its error.

erfc(z) = exp(-z^2) G(z).  G (the scaled complementary error function) is smooth and decays like
1 / (z sqrt(pi)); with t = 1 / (1 + z / 2) the quotient G / t is close to a low-degree polynomial in t.  The
script fits that polynomial (degree 8, weighted least squares on Chebyshev nodes, re-weighted until the relative
error is level), shifts it to powers of (t - t0) for a stable FP32 Horner evaluation, rounds the coefficients to
FP32, and then emulates the kernel's exact FP32 operation sequence (fused multiply-adds included) on 6e6 points
against the FP64 value of x erfc(-x / sqrt 2) / 2.

    python -m paper_2502_20853_amd.fit_gelu_erfcx

needs numpy and scipy; nothing at run time depends on it.
"""
import numpy as np
from scipy.special import erfc, erfcx

F32 = np.float32
P = 0.5
DEGREE = 8
ZMAX = 12.1


def fit():
    tmin = 1.0 / (1.0 + P * ZMAX)
    k = np.arange(6000)
    u = np.cos(np.pi * (k + 0.5) / 6000)
    t = (u * (1 - tmin) + (1 + tmin)) / 2
    g = erfcx((1 / t - 1) / P) / t
    V = np.polynomial.chebyshev.chebvander(u, DEGREE)
    w = np.ones_like(u)
    for _ in range(60):
        c, *_ = np.linalg.lstsq(V * (w / g)[:, None], w, rcond=None)
        rel = (V @ c) / g - 1
        w = w * (1 + 5 * np.abs(rel) / np.abs(rel).max())
        w /= w.mean()
    t0 = (1 + tmin) / 2
    mono = np.polynomial.chebyshev.Chebyshev(c, domain=[tmin, 1]).convert(kind=np.polynomial.Polynomial)
    shifted = np.polynomial.Polynomial(mono.coef)(np.polynomial.Polynomial([t0, 1.0]))
    return [float(F32(x)) for x in shifted.coef], float(F32(t0)), float(np.abs(rel).max())


def fma(a, b, c):
    return (a.astype(np.float64) * np.asarray(b, dtype=np.float64) + np.asarray(c, dtype=np.float64)).astype(F32)


def mul(a, b):
    return (a.astype(np.float64) * np.asarray(b, dtype=np.float64)).astype(F32)


def gelu_fp32(x, coef, t0):
    """The kernel's operation sequence, one FP32 rounding per operation."""
    l1 = float(F32(0.72134752044448170368))
    l2 = float(F32(0.72134752044448170368 - l1))
    x = x.astype(F32)
    ax = np.minimum(np.abs(x), F32(17.0))
    t = (F32(1) / fma(ax, float(F32(0.35355339059327376)), 1.0)).astype(F32)
    w = (t - F32(t0)).astype(F32)
    g = np.full_like(x, F32(coef[-1]))
    for c in coef[-2::-1]:
        g = fma(g, w, c)
    g = mul(g, t)
    s = mul(ax, ax)
    r = (ax.astype(np.float64) ** 2 - s.astype(np.float64)).astype(F32)
    yh = mul(s, l1)
    yl = (s.astype(np.float64) * l1 - yh.astype(np.float64)).astype(F32)
    yl = fma(s, l2, yl)
    e = np.exp2(-yh.astype(np.float64)).astype(F32)
    e = np.where(e < F32(1.1754944e-38), F32(0), e)            # results below the normal range are flushed
    c = fma(yl, -float(F32(np.log(2.0))), 1.0)
    c = fma(r, -0.5, c)
    h = mul(mul(mul(g, e), c), 0.5)
    return mul(x, np.where(x < 0, h, (F32(1) - h).astype(F32)))


def main():
    coef, t0, fit_err = fit()
    print("t0 =", repr(t0))
    for i, c in enumerate(coef):
        print("C%d = %r" % (i, c))
    print("relative error of the fit in exact arithmetic: %.2e" % fit_err)
    rng = np.random.default_rng(0)
    xs = np.concatenate([np.linspace(-17, 17, 2000001), rng.standard_normal(2000000) * 3,
                         -np.abs(rng.standard_normal(1000000)) * 6, rng.uniform(-14, -5, 1000000)])
    got = gelu_fp32(xs, coef, t0).astype(np.float64)
    x64 = xs.astype(F32).astype(np.float64)
    want = 0.5 * x64 * erfc(-x64 / np.sqrt(2.0))
    big = np.abs(want) >= 2.0 ** -100
    print("max |error| / |GELU| where |GELU| >= 2^-100: %.2e (2^-18 = %.2e)" % (
        (np.abs(got - want)[big] / np.abs(want)[big]).max(), 2.0 ** -18))
    print("max |error| elsewhere: %.2e (2^-120 = %.2e)" % (np.abs(got - want)[~big].max(), 2.0 ** -120))


if __name__ == "__main__":
    main()
