"""Pins for the CPU oracle: every check here compares the oracle with something
that is not the oracle's own formula -- values the paper prints, closed forms,
invariants, brute force, special cases that reduce to numpy routines."""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden")
PAPER = json.load(open(os.path.join(GOLD, "paper_worked_values.json")))
GRID = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
SIGNED_GRID = sorted(set([-g for g in GRID] + GRID))


def f32(x):
    return float(np.float32(x))


# ------------------------------------------------------------------ E2M1 ----

def test_e2m1_table_from_bit_fields(orc):
    # Sec. 3.1: 1 sign, 2 exponent, 1 mantissa bit; bias 1; Q_p = 6
    for code in range(16):
        s, e, m = code >> 3, (code >> 1) & 3, code & 1
        mag = m * 0.5 if e == 0 else (1 + m / 2) * 2.0 ** (e - 1)
        assert orc.e2m1_value(code) == (-mag if s else mag)
    vals = [orc.e2m1_value(c) for c in range(16)]
    assert max(vals) == PAPER["format"]["Qp"] and min(vals) == PAPER["format"]["Qn"]
    # largest binade starts at 2^E_max
    assert orc.e2m1_value(6) == 2.0 ** PAPER["emax"]["E_max"]


def test_threshold_example_adjacent_values(orc):
    # Sec. 4.1: -0.75 is the midpoint of the adjacent FP4 values -1 and -0.5
    t = PAPER["threshold_example"]
    vals = sorted(set(orc.e2m1_value(c) for c in range(16)))
    i = vals.index(t["q1"])
    assert vals[i + 1] == t["q2"] and (t["q1"] + t["q2"]) / 2 == t["thrd"]
    # just either side of the threshold; the threshold itself goes to q2 (strict <)
    assert orc.e2m1_value(orc.round_rtn(-0.7501)) == -1.0
    assert orc.e2m1_value(orc.round_rtn(-0.7499)) == -0.5
    assert orc.e2m1_value(orc.round_rtn(-0.75)) == -0.5


# --------------------------------------------------------- shared exponent --

def test_scale_worked_examples(orc):
    fl, tf = PAPER["floor_scale_example"], PAPER["truncfree_scale_example"]
    assert 2.0 ** orc.shared_exponent(fl["M"], orc.SCALE_FLOOR) == fl["S"]
    assert 2.0 ** orc.shared_exponent(tf["M"], orc.SCALE_TRUNCFREE) == tf["S"]
    # the whole quantizer on that group: 31 is stored as 6*4 under Eq. 2 and as 4*8 truncation-free
    x = np.zeros((1, 32), np.float32)
    x[0, 5] = 31.0
    x[0, 6] = -31.0
    c, s = orc.quantize(x, scale_mode=orc.SCALE_FLOOR)
    d = orc.dequantize(c, s)
    assert d[0, 5] == fl["stored_value_of_M"] * fl["S"] and d[0, 6] == -d[0, 5]
    c, s = orc.quantize(x, scale_mode=orc.SCALE_TRUNCFREE)
    d = orc.dequantize(c, s)
    assert s[0, 0] == 127 + 3 and d[0, 5] == 32.0 and d[0, 6] == -32.0  # 3.875 -> 4


def _exact_ceil_log2(fr):
    """ceil(log2(fr)) for a positive Fraction, by integer arithmetic only."""
    n, d = fr.numerator, fr.denominator
    s = n.bit_length() - d.bit_length()          # 2^(s-1) < fr < 2^(s+1)
    while Fraction(2) ** s < fr:
        s += 1
    while Fraction(2) ** (s - 1) >= fr:
        s -= 1
    return s


def _exact_floor_log2(fr):
    return -_exact_ceil_log2(1 / fr)


def test_shared_exponent_vs_exact_rational_and_bit_form(orc):
    rng = np.random.default_rng(1)
    bits = rng.integers(0x00800000, 0x7F000000, size=4000, dtype=np.uint32)
    # add values on and next to the 1.5 * 2^e boundary and exact powers of two
    special = []
    for e in range(-120, 120, 7):
        for m in (0x000000, 0x000001, 0x3FFFFF, 0x400000, 0x400001, 0x7FFFFF):
            special.append(((e + 127) << 23) | m)
    bits = np.concatenate([bits, np.array(special, np.uint32)])
    vals = bits.view(np.float32)
    for u, v in zip(bits.tolist(), vals.tolist()):
        fr = Fraction(v)
        tf = _exact_ceil_log2(fr / 6)
        fl = _exact_floor_log2(fr) - 2
        assert orc.shared_exponent(v, orc.SCALE_TRUNCFREE) == max(-127, min(127, tf))
        assert orc.shared_exponent(v, orc.SCALE_FLOOR) == max(-127, min(127, fl))
        # closed form on the FP32 fields: 6 = 1.5 * 2^2
        e, m = (u >> 23) - 127, u & 0x7FFFFF
        assert tf == e - 2 + (1 if m > 0x400000 else 0)
        assert fl == e - 2


def test_shared_exponent_edges(orc):
    # all-zero group: epsilon = 1e-8 -> ceil(log2(1e-8/6)) = floor(log2 1e-8) - 2 = -29
    eps = PAPER["zero_group_epsilon"]["epsilon"]
    assert math.ceil(math.log2(eps / 6)) == -29 and math.floor(math.log2(eps)) - 2 == -29
    assert orc.shared_exponent(0.0, orc.SCALE_TRUNCFREE) == -29
    assert orc.shared_exponent(0.0, orc.SCALE_FLOOR) == -29
    # |s| <= 127 (Sec. 3.1): smallest subnormal would need s = -151
    tiny = float(np.float32(1e-45))
    assert orc.shared_exponent(tiny, orc.SCALE_TRUNCFREE) == -127
    assert orc.shared_exponent(tiny, orc.SCALE_FLOOR) == -127
    big = float(np.finfo(np.float32).max)
    assert orc.shared_exponent(big, orc.SCALE_TRUNCFREE) == 126
    assert orc.shared_exponent(big, orc.SCALE_FLOOR) == 125
    # exactly 6 * 2^k sits at the top of the range, 2^k at the bottom of Eq. 2's
    assert orc.shared_exponent(6.0, orc.SCALE_TRUNCFREE) == 0
    assert orc.shared_exponent(f32(6.0000005), orc.SCALE_TRUNCFREE) == 1
    assert orc.shared_exponent(4.0, orc.SCALE_FLOOR) == 0
    assert orc.shared_exponent(f32(3.9999998), orc.SCALE_FLOOR) == -1


def test_range_invariants_per_group(orc):
    rng = np.random.default_rng(2)
    x = (rng.standard_normal((64, 256)) * np.exp(rng.uniform(-20, 20, (64, 1)))).astype(np.float32)
    M = np.abs(x.reshape(64, 8, 32)).max(-1).astype(np.float64)
    _, s = orc.quantize(x, scale_mode=orc.SCALE_TRUNCFREE)
    r = M / 2.0 ** (s.astype(np.int64) - 127)
    assert np.all(r <= 6.0) and np.all(r > 3.0)       # Q_n <= M/S <= Q_p, and the ceiling is tight
    _, s = orc.quantize(x, scale_mode=orc.SCALE_FLOOR)
    r = M / 2.0 ** (s.astype(np.int64) - 127)
    assert np.all(r >= 4.0) and np.all(r < 8.0)       # [2^Emax, 2^(Emax+1))


# -------------------------------------------------------------- round_D -----

def test_rtn_tie_vectors(orc):
    # strict "<" in round_D sends midpoints to q2, the upper neighbour
    ties = {0.25: 0.5, 0.75: 1.0, 1.25: 1.5, 1.75: 2.0, 2.5: 3.0, 3.5: 4.0, 5.0: 6.0,
            -0.25: 0.0, -0.75: -0.5, -1.25: -1.0, -1.75: -1.5, -2.5: -2.0, -3.5: -3.0, -5.0: -4.0}
    for y, q in ties.items():
        assert orc.e2m1_value(orc.round_rtn(y)) == q, y
    for g in SIGNED_GRID:                              # grid points are fixed points
        assert orc.e2m1_value(orc.round_rtn(g)) == g
    assert orc.round_rtn(-0.0) == 8 and orc.round_rtn(0.0) == 0
    assert orc.round_rtn(-0.1) == 8                    # sign bit follows the input


def test_rtn_brute_force_all_bf16(orc):
    # every bf16 value in [-6, 6]: nearest of the 15 values, ties to the larger value
    u = np.arange(65536, dtype=np.uint32) << 16
    y = u.view(np.float32)
    y = y[np.isfinite(y) & (np.abs(y) <= 6.0)]
    grid = np.array(SIGNED_GRID)
    for v in y.tolist():
        d = np.abs(grid - v)
        best = grid[np.flatnonzero(d == d.min()).max()]
        code = orc.round_rtn(v)
        assert orc.e2m1_value(code) == best, v
        assert (code >> 3) == (1 if math.copysign(1.0, v) < 0 else 0)


# -------------------------------------------------------------- round_S -----

def test_sr_exhaustive_counts(orc):
    # over all 65536 draws the larger magnitude is taken exactly ceil(65536 p) times
    for y in (0.1, 0.25, 0.3, 1.2, 1.999, 2.75, 4.5, 5.999, -0.3, -2.2, -5.0, 1e-6, 3.0, -6.0, 0.0):
        y = f32(y)
        a = abs(y)
        m1 = max(g for g in GRID if g <= a)
        m2 = min([g for g in GRID if g > m1] or [m1])
        p = Fraction(a) - Fraction(m1)
        p = p / Fraction(m2 - m1) if m2 > m1 else Fraction(0)
        ups = 0
        for r in range(65536):
            v = orc.e2m1_value(orc.round_sr(y, r))
            assert abs(v) in (m1, m2) and (v == 0 or (v < 0) == (y < 0))
            ups += abs(v) == m2 and m2 > m1
        assert ups == math.ceil(65536 * p), y
    assert orc.round_sr(-0.0, 0) == 8


def test_sr_extreme_draws(orc):
    assert orc.e2m1_value(orc.round_sr(f32(1e-30), 0)) == 0.5      # r = 0 rounds up iff p > 0
    assert orc.e2m1_value(orc.round_sr(2.0, 0)) == 2.0              # p = 0 never moves
    assert orc.e2m1_value(orc.round_sr(f32(2.99999), 65535)) == 3.0  # p > 65535/65536
    assert orc.e2m1_value(orc.round_sr(f32(2.9999), 65535)) == 2.0


def test_sr_unbiased_with_philox_stream(orc):
    # E[round_S(y)] = y (Sec. 3.2), driven by the real random stream
    n = 200000
    for y in (0.37, 1.1, 2.6, -4.9, -0.05):
        y = f32(y)
        acc = 0.0
        for e in range(n):
            acc += orc.e2m1_value(orc.round_sr(y, orc.sr_bits(123, 7, e)))
        a = abs(y)
        m1 = max(g for g in GRID if g <= a)
        m2 = min(g for g in GRID if g > m1)
        p = (a - m1) / (m2 - m1)
        tol = 5 * math.sqrt(p * (1 - p) / n) * (m2 - m1) + (m2 - m1) / 65536
        assert abs(acc / n - y) <= tol, (y, acc / n)


# --------------------------------------------------------------- Philox -----

def _philox_py(ctr, key):
    M0, M1, W0, W1 = 0xD2511F53, 0xCD9E8D57, 0x9E3779B9, 0xBB67AE85
    c = list(ctr)
    k = list(key)
    mask = 0xFFFFFFFF
    for _ in range(10):
        p0, p1 = M0 * c[0], M1 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & mask, (p0 >> 32) ^ c[3] ^ k[1], p0 & mask]
        k = [(k[0] + W0) & mask, (k[1] + W1) & mask]
    return c


def test_philox_known_answers(orc):
    kat = json.load(open(os.path.join(GOLD, "philox4x32_10_kat.json")))
    for v in kat["vectors"]:
        ctr = [int(x, 16) for x in v["ctr"]]
        key = [int(x, 16) for x in v["key"]]
        out = [int(x, 16) for x in v["out"]]
        assert orc.philox4x32_10(ctr, key) == out
        assert _philox_py(ctr, key) == out


def test_philox_vs_bigint_and_fields(orc):
    rng = np.random.default_rng(3)
    for _ in range(2000):
        ctr = [int(x) for x in rng.integers(0, 2**32, 4)]
        key = [int(x) for x in rng.integers(0, 2**32, 2)]
        assert orc.philox4x32_10(ctr, key) == _philox_py(ctr, key)
    # element e -> call e>>3, 16-bit field e&7, counting from the low half of word 0
    seed, tid = 0x1234567890ABCDEF, 42
    for e in (0, 1, 7, 8, 9, 12345, 2**35 + 5, 2**40 + 3):
        w = _philox_py([(e >> 3) & 0xFFFFFFFF, (e >> 3) >> 32, tid, 0], [seed & 0xFFFFFFFF, seed >> 32])
        j = e & 7
        assert orc.sr_bits(seed, tid, e) == (w[j >> 1] >> (16 * (j & 1))) & 0xFFFF
    # different tensor ids and seeds give different streams
    a = [orc.sr_bits(1, 1, e) for e in range(64)]
    assert a != [orc.sr_bits(1, 2, e) for e in range(64)]
    assert a != [orc.sr_bits(2, 1, e) for e in range(64)]


def test_philox_fields_uniform(orc):
    n = 1 << 16
    r = np.array([orc.sr_bits(5, 9, e) for e in range(n)])
    assert r.min() >= 0 and r.max() <= 65535
    hist = np.bincount(r >> 8, minlength=256)          # 256 bins, expect n/256 each
    chi2 = ((hist - n / 256) ** 2 / (n / 256)).sum()
    assert chi2 < 350                                  # 255 dof: mean 255, sd ~22.6
    assert abs(r.mean() - 32767.5) < 5 * 65536 / math.sqrt(12 * n)


# ------------------------------------------------------------ quantizers ----

def test_pack_layout_by_construction(orc):
    # a group that is already on the grid with max 6 -> s = 0 and codes known by hand
    mags = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    row = np.array(mags + [-m for m in mags] + mags + [-m for m in mags], np.float32)
    x = np.stack([row, row * 4.0, row[::-1] * 0.125])
    codes, scales = orc.quantize(x)
    assert scales.tolist() == [[127], [129], [124]]
    want0 = list(range(8)) + list(range(8, 16)) + list(range(8)) + list(range(8, 16))
    want = [want0, want0, want0[::-1]]
    for r in range(3):
        got = []
        for b in codes[r].tolist():
            got += [b & 15, b >> 4]                     # low nibble = even element
        assert got == want[r]
    assert np.array_equal(orc.dequantize(codes, scales), x.astype(np.float64))


def test_quantize_error_bound_and_scale_equivariance(orc):
    rng = np.random.default_rng(4)
    x = (rng.standard_normal((16, 128)) * np.exp(rng.uniform(-8, 8, (16, 128)))).astype(np.float32)
    for mode in (orc.SCALE_TRUNCFREE, orc.SCALE_FLOOR):
        codes, scales = orc.quantize(x, scale_mode=mode)
        S = np.repeat(2.0 ** (scales.astype(np.int64) - 127), 32, axis=1)
        y = x.astype(np.float64) / S
        if mode == orc.SCALE_FLOOR:
            assert np.abs(y).max() > 6.0               # Eq. 2 does overflow the range ...
            y = np.clip(y, -6, 6)                      # ... and truncates
        q = orc.dequantize(codes, scales) / S
        # nearest grid value: the error is at most half the local spacing
        spacing = np.where(np.abs(y) < 2, 0.5, np.where(np.abs(y) < 4, 1.0, 2.0))
        assert np.all(np.abs(q - y) <= spacing / 2)
        # multiplying by 2^7 moves every scale byte by 7 and no code
        c2, s2 = orc.quantize(x * np.float32(128.0), scale_mode=mode)
        assert np.array_equal(c2, codes) and np.array_equal(s2.astype(int), scales.astype(int) + 7)
        # SR result is one of the two neighbours of y
        c3, s3 = orc.quantize(x, round=orc.ROUND_SR, scale_mode=mode, seed=11, tensor_id=3)
        q3 = orc.dequantize(c3, s3) / S
        assert np.array_equal(s3, scales) and np.all(np.abs(q3 - y) < spacing + 1e-12)


def test_quantize_zero_group_and_ld(orc):
    x = np.zeros((2, 64), np.float32)
    x[1, 40] = -3.0
    codes, scales = orc.quantize(x)
    assert scales.tolist() == [[98, 98], [98, 127 - 1]]   # -29; 3/6 -> s = -1
    assert not codes[0].any() and orc.dequantize(codes, scales)[1, 40] == -3.0
    # a strided view gives the same bytes as its contiguous copy
    big = np.random.default_rng(5).standard_normal((8, 96)).astype(np.float32)
    v = big[:, 32:]
    a = orc.quantize(v, round=orc.ROUND_SR, seed=3, tensor_id=1)
    b = orc.quantize(np.ascontiguousarray(v), round=orc.ROUND_SR, seed=3, tensor_id=1)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_quotient_is_exact_below_fp32_range(orc):
    # x / S is a real quotient (Sec. 3.2): an element 2^-170 of the scale still has p > 0, so a
    # zero draw rounds it up, and the EMA rule still sees the bracket [0, 0.5] for it
    seed, tid = 4, 9
    e0 = next(e for e in range(1 << 20) if orc.sr_bits(seed, tid, e) == 0)
    x = np.zeros((1, ((e0 // 32) + 1) * 32), np.float32)
    x[0, (e0 // 32) * 32 + ((e0 + 1) % 32)] = np.float32(2.0) ** 20        # group maximum: s = 18
    x[0, e0] = np.float32(2.0) ** -149                                     # y = 2^-167
    codes, scales = orc.quantize(x, round=orc.ROUND_SR, seed=seed, tensor_id=tid)
    assert scales[0, e0 // 32] == 127 + 18
    assert (codes[0, e0 // 2] >> (4 * (e0 & 1))) & 15 == 1                  # 0.5 * S
    xn = -x
    codes, _ = orc.quantize(xn, round=orc.ROUND_SR, seed=seed, tensor_id=tid)
    assert (codes[0, e0 // 2] >> (4 * (e0 & 1))) & 15 == 9
    codes, _ = orc.quantize(x, round=orc.ROUND_RTN)
    assert (codes[0, e0 // 2] >> (4 * (e0 & 1))) & 15 == 0
    ema = x.copy()
    ema[0, e0] = np.float32(2.0) ** 17                                     # z = 0.5: pulls the tiny weight up
    codes, _ = orc.ema_weight_quant(x, ema, update_ema=0)
    assert (codes[0, e0 // 2] >> (4 * (e0 & 1))) & 15 == 1


def test_quantize_sr_decisions_follow_element_index(orc):
    # compose the whole quantizer from its pinned parts on a small matrix
    rng = np.random.default_rng(6)
    x = rng.standard_normal((4, 64)).astype(np.float32)
    seed, tid, base = 99, 5, 8 * 1000
    codes, scales = orc.quantize(x, round=orc.ROUND_SR, seed=seed, tensor_id=tid, index_base=base)
    for r in range(4):
        for c in range(64):
            s = int(scales[r, c // 32]) - 127
            y = f32(np.ldexp(x[r, c], -s))
            want = orc.round_sr(y, orc.sr_bits(seed, tid, base + r * 64 + c))
            got = (codes[r, c // 2] >> (4 * (c & 1))) & 15
            assert got == want


def test_transposed_reduces_to_row_quantizer_of_transpose(orc):
    rng = np.random.default_rng(7)
    x = (rng.standard_normal((64, 96)) * 3).astype(np.float32)
    ct, st, _, _ = orc.quantize_transposed(x, round_t=orc.ROUND_RTN, pre_quant=0, want_row=False)
    c, s = orc.quantize(np.ascontiguousarray(x.T))
    assert ct.shape == (96, 32) and st.shape == (96, 2)
    assert np.array_equal(ct, c) and np.array_equal(st, s)


def test_transposed_sr_uses_source_index(orc):
    rng = np.random.default_rng(8)
    x = rng.standard_normal((32, 40)).astype(np.float32)
    seed, tid, base = 7, 6, 64
    ct, st, _, _ = orc.quantize_transposed(x, round_t=orc.ROUND_SR, tensor_id_t=tid, pre_quant=0,
                                           want_row=False, seed=seed, index_base=base)
    for c in range(40):
        s = int(st[c, 0]) - 127
        for i in range(32):
            y = f32(np.ldexp(x[i, c], -s))
            want = orc.round_sr(y, orc.sr_bits(seed, tid, base + i * 40 + c))
            assert (ct[c, i // 2] >> (4 * (i & 1))) & 15 == want


def test_double_quantization_is_composition(orc):
    rng = np.random.default_rng(9)
    x = (rng.standard_normal((64, 64)) * 2).astype(np.float32)
    x[:, 3] *= 20
    ct, st, cr, sr = orc.quantize_transposed(x, round_t=orc.ROUND_SR, tensor_id_t=6, pre_quant=1,
                                             round_row=orc.ROUND_RTN, tensor_id_row=1, seed=5)
    c1, s1 = orc.quantize(x)
    assert np.array_equal(cr, c1) and np.array_equal(sr, s1)
    xq = orc.dequantize(c1, s1).astype(np.float32)
    ct2, st2, _, _ = orc.quantize_transposed(xq, round_t=orc.ROUND_SR, tensor_id_t=6, pre_quant=0,
                                             want_row=False, seed=5)
    assert np.array_equal(ct, ct2) and np.array_equal(st, st2)
    # handing the row result in gives the same bytes
    ct3, st3, _, _ = orc.quantize_transposed(x, round_t=orc.ROUND_SR, tensor_id_t=6, pre_quant=1,
                                             want_row=False, row_in=(c1, s1), seed=5)
    assert np.array_equal(ct, ct3) and np.array_equal(st, st3)
    # without double quantization the result differs (Microscaling's design, Eqs. 6-7)
    ct4, _, _, _ = orc.quantize_transposed(x, round_t=orc.ROUND_SR, tensor_id_t=6, pre_quant=0,
                                           want_row=False, seed=5)
    assert not np.array_equal(ct, ct4)


# ----------------------------------------------------------------- Q-EMA ----

def test_qema_equals_rtn_when_ema_is_weight(orc):
    rng = np.random.default_rng(10)
    w = (rng.standard_normal((32, 128)) * 0.02).astype(np.float32)
    ema = np.zeros_like(w)
    c, s = orc.ema_weight_quant(w, ema, update_ema=2)
    c0, s0 = orc.quantize(w)
    assert np.array_equal(ema, w) and np.array_equal(c, c0) and np.array_equal(s, s0)
    ema = rng.standard_normal(w.shape).astype(np.float32)
    c, s = orc.ema_weight_quant(w, ema, beta=0.0, update_ema=1)   # beta = 0: ema <- w
    assert np.array_equal(ema, w) and np.array_equal(c, c0)


def test_qema_micro_example_and_bracket(orc):
    # around the -0.75 threshold of Sec. 4.1: latent -0.74 alone rounds to -0.5,
    # an EMA latent of -0.80 pulls it to -1
    assert orc.e2m1_value(orc.round_rtn(f32(-0.74))) == -0.5
    assert orc.e2m1_value(orc.round_ema(f32(-0.74), f32(-0.80))) == -1.0
    assert orc.e2m1_value(orc.round_ema(f32(-0.74), f32(-0.70))) == -0.5
    assert orc.e2m1_value(orc.round_ema(f32(-0.74), f32(-0.75))) == -0.5   # tie -> q2
    assert orc.e2m1_value(orc.round_ema(f32(0.74), f32(0.75))) == 1.0      # tie -> q2
    # EMA outside the bracket picks the nearer end; never leaves the bracket of w/S
    assert orc.e2m1_value(orc.round_ema(f32(2.2), f32(-5.0))) == 2.0
    assert orc.e2m1_value(orc.round_ema(f32(2.2), f32(5.0))) == 3.0
    assert orc.round_ema(f32(-0.3), f32(4.0)) == 8                         # -0
    # a latent weight that is already an E2M1 value stays
    for g in SIGNED_GRID:
        assert orc.e2m1_value(orc.round_ema(g, 100.0)) == g
        assert orc.e2m1_value(orc.round_ema(g, -100.0)) == g
    rng = np.random.default_rng(11)
    w = (rng.standard_normal((16, 64)) * 0.02).astype(np.float32)
    ema = (w + rng.standard_normal(w.shape).astype(np.float32) * 0.004).astype(np.float32)
    c, s = orc.ema_weight_quant(w, ema.copy(), update_ema=0)
    c0, s0 = orc.quantize(w)
    assert np.array_equal(s, s0)
    S = np.repeat(2.0 ** (s.astype(np.int64) - 127), 32, axis=1)
    y = w / S
    q = orc.dequantize(c, s) / S
    lo = np.array([max(g for g in SIGNED_GRID if g <= v) for v in y.ravel()]).reshape(y.shape)
    hi = np.array([min(g for g in SIGNED_GRID if g >= v) for v in y.ravel()]).reshape(y.shape)
    assert np.all((q == lo) | (q == hi))
    z = ema / S
    pick_hi = np.abs(z - lo) >= np.abs(z - hi)
    assert np.array_equal(q, np.where(pick_hi, hi, lo))
    assert not np.array_equal(c, c0)                   # and it does differ from plain RTN


def test_ema_update_closed_form(orc):
    # constant weight: ema_t = w + beta^t (ema_0 - w)
    beta = PAPER["ema_beta"]["beta"]
    w = np.full((1, 32), 0.5, np.float32)
    ema = np.full((1, 32), -1.0, np.float32)
    for _ in range(50):
        orc.ema_weight_quant(w, ema, beta=beta, update_ema=1)
    want = 0.5 + f32(beta) ** 50 * (-1.5)
    assert np.allclose(ema, want, rtol=0, atol=2e-6)
    e0 = ema.copy()
    orc.ema_weight_quant(w, ema, beta=beta, update_ema=0)
    assert np.array_equal(ema, e0)


# ------------------------------------------------------------------ GEMM ----

def test_gemm_vs_numpy_and_structure(orc):
    rng = np.random.default_rng(12)
    A = rng.standard_normal((5, 96)).astype(np.float32) * 3
    B = rng.standard_normal((7, 96)).astype(np.float32) * 0.02
    ac, as_ = orc.quantize(A)
    bc, bs = orc.quantize(B)
    C = orc.gemm_f64(ac, as_, bc, bs)
    ref = orc.dequantize(ac, as_) @ orc.dequantize(bc, bs).T
    assert C.shape == (5, 7) and np.allclose(C, ref, rtol=1e-13, atol=0)
    # adding 1 to every scale byte of A doubles C exactly
    C2 = orc.gemm_f64(ac, as_ + 1, bc, bs)
    assert np.array_equal(C2, 2 * C)
    ii = np.array([0, 4, 2, 3])
    jj = np.array([6, 0, 5, 3])
    v, av = orc.gemm_f64_sampled(ac, as_, bc, bs, ii, jj)
    assert np.array_equal(v, C[ii, jj])
    aref = np.abs(orc.dequantize(ac, as_)) @ np.abs(orc.dequantize(bc, bs)).T
    assert np.allclose(av, aref[ii, jj], rtol=1e-13)


def test_gemm_one_hot_by_hand(orc):
    # A row i has a single 3 at k = 10*i+1, B row j a single -2 at k = 10*j+1, scales 2^1 and 2^-2
    m, n, k = 3, 4, 64
    ac = np.zeros((m, k // 2), np.uint8)
    bc = np.zeros((n, k // 2), np.uint8)
    for i in range(m):
        ac[i, (10 * i + 1) // 2] = 5 << 4                # code 5 = 3.0 in the high nibble (odd k)
    for j in range(n):
        bc[j, (10 * j + 1) // 2] = 12 << 4               # code 12 = -2.0
    as_ = np.full((m, 2), 128, np.uint8)
    bs = np.full((n, 2), 125, np.uint8)
    C = orc.gemm_f64(ac, as_, bc, bs)
    want = np.zeros((m, n))
    for i in range(min(m, n)):
        want[i, i] = (3 * 2) * (-2 * 0.25)
    assert np.array_equal(C, want)


def test_layer_gradients_unbiased(orc):
    # Sec. 3.4: E[Q3(dY) Q4(Q2(W))] = dY Q2(W) and E[Q5(dY^T) Q6(Q1(X))] = dY^T Q1(X)
    rng = np.random.default_rng(13)
    N = D = C = 32
    X = rng.standard_normal((N, D)).astype(np.float32)
    W = (rng.standard_normal((C, D)) * 0.02).astype(np.float32)
    dY = (rng.standard_t(3, (N, C)) * 1e-3).astype(np.float32)
    xq = orc.dequantize(*orc.quantize(X))
    wq = orc.dequantize(*orc.quantize(W))
    dX_ref = dY.astype(np.float64) @ wq
    dW_ref = dY.astype(np.float64).T @ xq
    trials = 300
    dX = np.zeros((N, D))
    dW = np.zeros((C, D))
    sqX = np.zeros((N, D))
    sqW = np.zeros((C, D))
    for t in range(trials):
        seed = 1000 + t
        dyT_c, dyT_s, dy_c, dy_s = orc.quantize_transposed(
            dY, round_t=orc.ROUND_SR, tensor_id_t=5, pre_quant=0, round_row=orc.ROUND_SR,
            tensor_id_row=3, seed=seed)
        wT_c, wT_s, _, _ = orc.quantize_transposed(W, round_t=orc.ROUND_SR, tensor_id_t=4, pre_quant=1,
                                                   want_row=False, seed=seed)
        xT_c, xT_s, _, _ = orc.quantize_transposed(X, round_t=orc.ROUND_SR, tensor_id_t=6, pre_quant=1,
                                                   want_row=False, seed=seed)
        a = orc.gemm_f64(dy_c, dy_s, wT_c, wT_s)        # dX = Q3(dY) . Q4(...)   [N x D], K = C
        b = orc.gemm_f64(dyT_c, dyT_s, xT_c, xT_s)      # dW = Q5(dY^T) . Q6(...) [C x D], K = N
        dX += a
        dW += b
        sqX += a * a
        sqW += b * b
    for mean, sq, ref in ((dX / trials, sqX / trials, dX_ref), (dW / trials, sqW / trials, dW_ref)):
        sd = np.sqrt(np.maximum(sq - mean * mean, 0) / trials)
        zscore = np.abs(mean - ref) / (sd + 1e-12 * np.abs(ref).max())
        assert zscore.max() < 6.0 and np.mean(zscore < 3.0) > 0.98
    # the deterministic Microscaling flow (Eqs. 6-7) is visibly biased on the same data
    dyq = orc.dequantize(*orc.quantize(dY))
    wT_c, wT_s, _, _ = orc.quantize_transposed(W, round_t=orc.ROUND_RTN, pre_quant=0, want_row=False)
    bias = np.abs(dyq @ orc.dequantize(wT_c, wT_s).T - dX_ref).mean()
    assert bias > 3 * np.abs(dX / trials - dX_ref).mean()


# ------------------------------------------------- Q-Ramping: oscillation detection ----

def _osc_state(shape):
    return {k: np.zeros(shape, np.float32) for k in ("w_prev", "wq_prev", "dist_w", "dist_q")}


def test_oscillation_distances_closed_forms(orc):
    # Sec. 6.1: dist_W = sum |w^t - w^(t-1)|, dist_Q = sum |w_Q^t - w_Q^(t-1)|.
    # Row 0 drifts by 2^-10 per step (every partial sum exact in FP32): dist_W = T * 2^-10.
    # Row 1 holds an element whose latent weight w/S hops between -0.76 and -0.74 around the
    # threshold -0.75 of Sec. 4.1: its quantized value flips between -1 and -0.5 times S on
    # every step, so each step adds |q1 - q2| * S = 0.5 * S to dist_Q, and 0.02 * S to dist_W.
    T, S = 12, 0.25
    base = np.zeros((2, 32), np.float32)
    base[0, :] = np.linspace(0.5, 1.5, 32, dtype=np.float32)
    base[1, 0] = 6.0 * S                   # fixes the group's scale: M/S = 6 exactly
    st = _osc_state(base.shape)
    for t in range(T + 1):
        w = base.copy()
        w[0, :] += np.float32(t * 2.0 ** -10)
        w[1, 1] = np.float32((-0.76 if t % 2 == 0 else -0.74) * S)
        codes, scales = orc.quantize(w)
        assert scales[1, 0] == 127 - 2     # S = 2^-2
        orc.oscillation_accumulate(w, codes, scales, st, init=(t == 0))
    assert np.all(st["dist_w"][0] == np.float32(T * 2.0 ** -10))
    q = orc.dequantize(codes, scales)
    assert q[1, 1] in (-1.0 * S, -0.5 * S)
    assert st["dist_q"][1, 1] == np.float32(T * 0.5 * S)
    assert abs(st["dist_w"][1, 1] - T * 0.02 * S) < 1e-6
    assert st["dist_q"][1, 0] == 0.0 and st["dist_w"][1, 0] == 0.0          # an element that never moves
    # the oscillating element has R_w = 25, the drifting ones R_w <= a few
    R = st["dist_q"][1, 1] / st["dist_w"][1, 1]
    assert abs(R - 25.0) < 1e-3
    assert np.all(orc.ramping_factor(st["dist_w"], st["dist_q"], 16.0, 5, 16)[1, 1] == 6)


def test_oscillation_window_restart_and_independent_formulation(orc):
    # the same sums with numpy on dequantized weights (FP32 differences, FP32 running sums)
    import mx_workloads as wl
    st = _osc_state((96, 64))
    prev_w = prev_q = None
    dw = np.zeros((96, 64), np.float32)
    dq = np.zeros((96, 64), np.float32)
    for t, W in enumerate(wl.weight_walk(96, 64, seed=3, steps=6, sigma=2e-3)):
        codes, scales = orc.quantize(W)
        q = orc.dequantize(codes, scales).astype(np.float32)
        restart = t in (0, 4)              # a new detection window at step 4
        orc.oscillation_accumulate(W, codes, scales, st, init=restart)
        if restart:
            dw[:] = 0
            dq[:] = 0
        else:
            dw = (dw + np.abs(W - prev_w)).astype(np.float32)
            dq = (dq + np.abs(q - prev_q)).astype(np.float32)
        prev_w, prev_q = W.copy(), q.copy()
        assert np.array_equal(st["dist_w"], dw) and np.array_equal(st["dist_q"], dq)
        assert np.array_equal(st["w_prev"], W) and np.array_equal(st["wq_prev"], q)
    assert dq.max() > 0 and dw.min() > 0


def test_ramping_factor_formula(orc):
    # Algorithm 2 with the paper's defaults k1 = 16, k2 = 5
    g = PAPER["q_ramping"]
    for ex in g["factor_examples"]:
        got = orc.ramping_factor(np.array([[1.0]], np.float32), np.array([[ex["R"]]], np.float32), g["k1"], g["k2"], 64)
        assert got[0, 0] == ex["N"], ex
    # cap, and the degenerate trajectories
    assert orc.ramping_factor(np.array([[1.0]], np.float32), np.array([[1e6]], np.float32), 16, 5, 16)[0, 0] == 16
    assert orc.ramping_factor(np.array([[0.0]], np.float32), np.array([[0.0]], np.float32), 16, 5, 16)[0, 0] == 1
    assert orc.ramping_factor(np.array([[0.0]], np.float32), np.array([[0.5]], np.float32), 16, 5, 16)[0, 0] == 16
    # brute force over a grid of ratios with exact rational arithmetic
    rng = np.random.default_rng(0)
    dw = rng.integers(1, 1000, 500).astype(np.float32)
    dq = rng.integers(0, 100000, 500).astype(np.float32)
    got = orc.ramping_factor(dw.reshape(1, -1), dq.reshape(1, -1), 16, 5, 40).ravel()
    for a, b, n in zip(dw, dq, got):
        r = np.float32(b) / np.float32(a)                    # the FP32 quotient the definition uses
        want = min(5 * math.floor(Fraction(float(r)) / 16) + 1, 40)
        assert n == want


# ------------------------------------------------- oscillation diagnostics ----

def _latent_group(latents, S=0.25):
    """One 1x32 group whose scale is S (an element at 6*S pins it) holding the given latent values."""
    assert len(latents) <= 31
    w = np.zeros((1, 32), np.float32)
    w[0, 0] = 6.0 * S
    w[0, 1:1 + len(latents)] = np.asarray(latents, np.float64) * S
    return w


def test_quant_confidence_thresholds_and_cell_centres(orc):
    # Sec. 4.2: 0 on a threshold (a midpoint of neighbouring FP4 values, e.g. the -0.75 of Sec. 4.1),
    # 1 where the latent value is as far from every threshold as its FP4 value allows.
    thr = [(a + b) / 2 for a, b in zip(SIGNED_GRID[:-1], SIGNED_GRID[1:])]
    assert PAPER["threshold_example"]["thrd"] in thr and len(thr) == 14
    conf = orc.quant_confidence(_latent_group(thr))
    assert np.all(conf[0, 1:15] == 0.0)
    # the furthest points: midway between the two thresholds of a cell; +-6 for the outermost cells
    far = [0.0, 0.5, -0.5, 1.0, -1.0, 1.5, -1.5, 2.125, -2.125, 3.0, -3.0, 4.25, -4.25, 6.0, -6.0]
    conf = orc.quant_confidence(_latent_group(far))
    assert np.all(conf[0, 1:16] == 1.0) and conf[0, 0] == 1.0
    # values in between, by hand: cell of 2 is [1.75, 2.5], of 4 is [3.5, 5], of 6 is [5, 6], of 0 is [-.25, .25]
    by_hand = {2.0: 0.25 / 0.375, 4.0: 0.5 / 0.75, -4.0: 0.5 / 0.75, 5.5: 0.5, -5.25: 0.25, 0.125: 0.5,
               0.375: 0.5, 2.25: 0.25 / 0.375, 3.25: 0.5, 1.125: 0.5}
    conf = orc.quant_confidence(_latent_group(list(by_hand)))
    for i, (y, c) in enumerate(by_hand.items()):
        assert conf[0, 1 + i] == np.float32(c), (y, conf[0, 1 + i], c)


def test_quant_confidence_brute_force_definition(orc):
    # the definition taken literally, in rationals: MaxDist(v) by scanning every latent value on a
    # 1/64 grid of [-6, 6] (thresholds and cell centres are multiples of 1/8), min over all thresholds
    thr = [Fraction(a + b) / 2 for a, b in zip(SIGNED_GRID[:-1], SIGNED_GRID[1:])]
    grid = [Fraction(v) for v in SIGNED_GRID]

    def nearest(y):                      # round_D: ties toward the larger value
        best = min(abs(y - g) for g in grid)
        return max(g for g in grid if abs(y - g) == best)

    maxdist = {}
    for k in range(-6 * 64, 6 * 64 + 1):
        y = Fraction(k, 64)
        d = min(abs(y - t) for t in thr)
        v = nearest(y)
        maxdist[v] = max(maxdist.get(v, Fraction(0)), d)
    rng = np.random.default_rng(11)
    w = (rng.standard_normal((6, 64)) * rng.choice([1e-3, 0.02, 1.0, 30.0], (6, 1))).astype(np.float32)
    for mode in (orc.SCALE_TRUNCFREE, orc.SCALE_FLOOR):
        conf = orc.quant_confidence(w, mode)
        codes, scales = orc.quantize(w, orc.ROUND_RTN, mode)
        assert conf.min() >= 0.0 and conf.max() <= 1.0
        for r in range(w.shape[0]):
            for c in range(w.shape[1]):
                S = Fraction(2) ** (int(scales[r, c // 32]) - 127)
                y = Fraction(float(w[r, c])) / S
                y = max(min(y, Fraction(6)), Fraction(-6))          # Eq. 2's scale can overflow: clipped
                q = min(abs(y - t) for t in thr) / maxdist[nearest(y)]
                got = Fraction(float(conf[r, c]))
                half_ulp = Fraction(float(np.spacing(np.float32(max(float(q), 2.0 ** -126))))) / 2
                assert abs(got - q) <= half_ulp, (r, c, float(y), float(got), float(q))


def test_quant_confidence_invariances_and_histogram(orc):
    import mx_workloads as wl
    w = wl.weights(64, 96, seed=21)
    conf, hist = orc.quant_confidence(w, bins=20)
    assert np.array_equal(conf, orc.quant_confidence(w))
    # a power-of-two rescale moves weight and thresholds alike; so does a sign flip
    assert np.array_equal(conf, orc.quant_confidence(w * np.float32(2.0 ** -7)))
    assert np.array_equal(conf, orc.quant_confidence(-w))
    assert hist.sum() == w.size
    ref = np.bincount(np.minimum(19, np.floor(conf * np.float32(20)).astype(np.int64)).ravel(), minlength=20)
    assert np.array_equal(hist, ref.astype(np.uint64))
    # an all-zero group has latent value 0 everywhere: confidence 1
    z = np.zeros((1, 32), np.float32)
    assert np.all(orc.quant_confidence(z) == 1.0)
    # a strided source reads the same values
    big = np.zeros((64, 128), np.float32)
    big[:, :96] = w
    assert np.array_equal(orc.quant_confidence(big[:, :96]), conf)


def test_rate_of_change_closed_forms_and_numpy(orc):
    # Sec. 4.1: one term ||X^t - X^(t-1)||_F / ||X^(t-1)||_F
    rng = np.random.default_rng(5)
    prev = (rng.integers(-512, 512, (48, 40)) / 64.0).astype(np.float32)
    prev[0, 0] = 1.0
    # X^t = 1.5 X^(t-1): every product exact, ratio exactly 0.5 up to the rounding of the sums
    xp = prev.copy()
    r = orc.rate_of_change_term((1.5 * prev).astype(np.float32), xp)
    assert abs(r - 0.5) < 1e-14
    assert np.array_equal(xp, (1.5 * prev).astype(np.float32))           # the previous tensor is replaced
    # no change: 0
    assert orc.rate_of_change_term(xp.copy(), xp) == 0.0
    # one element moved by d: ||dX|| = |d|
    x = prev.copy()
    x[3, 7] += np.float32(0.25)
    xp = prev.copy()
    r = orc.rate_of_change_term(x, xp)
    assert abs(r - 0.25 / np.linalg.norm(prev.astype(np.float64))) < 1e-15
    # library norms on random data, strided source
    a = rng.standard_normal((80, 96)).astype(np.float32)
    b = (a + 1e-3 * rng.standard_normal((80, 96))).astype(np.float32)
    big = np.zeros((80, 160), np.float32)
    big[:, :96] = b
    xp = a.copy()
    r = orc.rate_of_change_term(big[:, :96], xp)
    ref = np.linalg.norm(b.astype(np.float64) - a.astype(np.float64)) / np.linalg.norm(a.astype(np.float64))
    assert abs(r - ref) <= 1e-13 * ref
    assert np.array_equal(xp, b)
    # a zero previous tensor: 0/0 reads 0, d/0 reads infinity
    z = np.zeros((2, 32), np.float32)
    assert orc.rate_of_change_term(z.copy(), z.copy()) == 0.0
    assert orc.rate_of_change_term(np.ones((2, 32), np.float32), z.copy()) == math.inf
    # the average over a window is r(X): a tensor that doubles every step has r = 1
    xp = prev.copy()
    terms = [orc.rate_of_change_term((prev * np.float32(2.0 ** (t + 1))), xp) for t in range(5)]
    assert abs(sum(terms) / 5 - 1.0) < 1e-14


# ------------------------------------------------- Q-Ramping's customised AdamW ----

def _torch_adamw_run(w0, grads, lr, betas, eps, wd):
    """torch.optim.AdamW (CPU, FP64, plain single-tensor path) over a list of gradients."""
    import torch
    p = torch.nn.Parameter(torch.tensor(np.asarray(w0, np.float64)))
    opt = torch.optim.AdamW([p], lr=lr, betas=betas, eps=eps, weight_decay=wd, foreach=False)
    out = []
    for g in grads:
        p.grad = torch.tensor(np.asarray(g, np.float64))
        opt.step()
        out.append(p.detach().numpy().copy())
    return out


def test_ramping_adamw_factor_one_is_adamw(orc):
    # Algorithm 2 with N_w = 1 everywhere is "normal AdamW": the library's, step for step
    rng = np.random.default_rng(3)
    w0 = rng.standard_normal(257) * 0.05
    grads = [rng.standard_normal(257) * 10.0 ** rng.uniform(-4, 0) for _ in range(12)]
    hp = dict(lr=2e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.05)
    ref = _torch_adamw_run(w0, grads, hp["lr"], (hp["beta1"], hp["beta2"]), hp["eps"], hp["weight_decay"])
    for factor in (None, np.ones(257, np.int32)):
        st = orc.ramping_adamw_state(w0)
        for t, g in enumerate(grads):
            orc.ramping_adamw_step(st, g, factor, **hp)
            assert np.allclose(st["w"], ref[t], rtol=1e-12, atol=1e-15), t
            assert np.all(st["updates"] == t + 1) and np.all(st["acc_steps"] == 0) and np.all(st["g_acc"] == 0)


def test_ramping_adamw_element_follows_large_batch_adamw(orc):
    # Sec. 6.2: an element with factor N has N times the batch size (its gradients are accumulated
    # over N steps) and N times the learning rate.  So it must follow AdamW at lr * N on the means
    # of N consecutive gradients, and stand still in between; elements are independent.
    rng = np.random.default_rng(4)
    n, T = 60, 24
    w0 = rng.standard_normal(n) * 0.05
    grads = [rng.standard_normal(n) * 0.01 for _ in range(T)]
    factor = np.array([1, 2, 3, 4, 6, 16] * 10, np.int32)
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    st = orc.ramping_adamw_state(w0)
    traj = []
    for g in grads:
        orc.ramping_adamw_step(st, g, factor, **hp)
        traj.append(st["w"].copy())
    for N in (1, 2, 3, 4, 6, 16):
        sel = factor == N
        means = [np.mean(grads[k * N:(k + 1) * N], axis=0)[sel] for k in range(T // N)]
        ref = _torch_adamw_run(w0[sel], means, hp["lr"] * N, (hp["beta1"], hp["beta2"]), hp["eps"], hp["weight_decay"])
        for t in range(T):
            done = (t + 1) // N                       # updates made after step t (0-based)
            want = w0[sel] if done == 0 else ref[done - 1]
            assert np.allclose(traj[t][sel], want, rtol=1e-12, atol=1e-15), (N, t)
        assert np.all(st["updates"][sel] == T // N)
        assert np.all(st["acc_steps"][sel] == T % N)


def test_ramping_adamw_first_update_closed_form_and_refactor(orc):
    # First AdamW update without decay: m_hat = g, v_hat = g^2, so w moves by lr_w * g / (|g| + eps):
    # N * lr in the direction opposite to the mean gradient.
    w0 = np.array([1.0, -2.0, 0.5, 0.25])
    factor = np.array([1, 4, 4, 2], np.int32)
    g = np.array([0.3, -0.2, 0.1, 0.0])
    st = orc.ramping_adamw_state(w0)
    for t in range(4):
        orc.ramping_adamw_step(st, g, factor, lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0)
        if t == 0:
            assert abs(st["w"][0] - (1.0 - 1e-2)) < 1e-9
            assert st["w"][1] == -2.0 and st["w"][2] == 0.5       # their batches are not full
            assert np.all(st["m"][1:] == 0) and np.all(st["v"][1:] == 0)
            assert list(st["acc_steps"]) == [0, 1, 1, 1]
    assert abs(st["w"][1] - (-2.0 + 4e-2)) < 1e-8                  # one update of 4 * lr against the sign of g
    assert abs(st["w"][2] - (0.5 - 4e-2)) < 1e-8
    assert st["w"][3] == 0.25                                      # zero gradient: 0 / (0 + eps) = 0
    assert list(st["updates"]) == [4, 1, 1, 2]
    # a new detection lowers an element's factor below what it has accumulated: it updates at once,
    # with the mean of what it holds
    st = orc.ramping_adamw_state([0.0])
    for gval in (1.0, 2.0, 3.0):
        orc.ramping_adamw_step(st, [gval], np.array([8], np.int32), lr=1e-2, weight_decay=0.0)
    assert st["updates"][0] == 0 and st["g_acc"][0] == 6.0
    orc.ramping_adamw_step(st, [6.0], np.array([2], np.int32), lr=1e-2, weight_decay=0.0)
    assert st["updates"][0] == 1 and st["acc_steps"][0] == 0
    assert abs(st["m"][0] - 0.1 * 3.0) < 1e-15                     # mean of 1, 2, 3, 6
    assert abs(st["w"][0] - (-2e-2)) < 1e-9                        # lr_w = 2 * lr


# ------------------------------------------------------------- column sums (bias gradient) ----

def test_column_sums_closed_forms(orc):
    """Values fixed by arithmetic: x[r][c] = c + 1 sums to rows * (c + 1); x[r][c] = r to rows(rows-1)/2;
    a sign alternating down the rows cancels (even row count) or leaves one term (odd); one element
    alone; a strided view sums its own columns only; FP64 keeps what FP32 accumulation would lose."""
    rows, cols = 37, 64
    c1 = np.tile(np.arange(1, cols + 1, dtype=np.float32), (rows, 1))
    assert np.array_equal(orc.column_sums(c1), rows * np.arange(1, cols + 1, dtype=np.float64))
    r1 = np.tile(np.arange(rows, dtype=np.float32)[:, None], (1, cols))
    assert np.array_equal(orc.column_sums(r1), np.full(cols, rows * (rows - 1) / 2.0))
    alt = np.where(np.arange(rows)[:, None] % 2 == 0, 1.0, -1.0).astype(np.float32) * np.arange(1, cols + 1, dtype=np.float32)
    assert np.array_equal(orc.column_sums(alt), np.arange(1, cols + 1, dtype=np.float64))       # 37 rows: one term left
    assert np.array_equal(orc.column_sums(alt[:36]), np.zeros(cols))
    one = np.zeros((rows, cols), np.float32)
    one[29, 5] = -2.5
    want = np.zeros(cols)
    want[5] = -2.5
    assert np.array_equal(orc.column_sums(one), want)
    wide = np.arange(rows * 2 * cols, dtype=np.float32).reshape(rows, 2 * cols)
    left = orc.column_sums(wide[:, :cols])
    assert np.array_equal(left, (np.arange(rows, dtype=np.float64)[:, None] * 2 * cols + np.arange(cols)).sum(0))
    big = np.full((4097, 32), 1.0, np.float32)
    big[0] = 2.0 ** 25                                   # in FP32, 2^25 + 1 = 2^25: 4096 ones would vanish
    assert np.array_equal(orc.column_sums(big), np.full(32, 2.0 ** 25 + 4096))


def test_column_sums_f32_ordered_pins(orc):
    """The FP32 fixed-order sums: exact (equal to the FP64 sums) whenever every partial sum is an integer
    below 2^24; on values built so that the order of the additions decides the result they give what the
    documented order gives, worked out by hand, and not what index order would give."""
    rng = np.random.default_rng(3)
    for rows in (32, 288, 2080):
        x = rng.integers(-64, 64, (rows, 40)).astype(np.float32)
        assert np.array_equal(orc.column_sums_f32_ordered(x).astype(np.float64), orc.column_sums(x))
    # one tile: rows 0..3 hold 2^24, 1, 1, 1 -> ((2^24 + 1) + 1) + 1 = 2^24 in FP32 (each +1 is a tie to even);
    # rows 4..7 hold 1, 1, 1, 1 -> 4; the tree then adds 2^24 + 4 exactly.  Index order from row 4 on would
    # give the same, but starting the rows 4..7 before the rows 0..3 would not: the value pins the grouping.
    x = np.zeros((32, 1), np.float32)
    x[0, 0] = 2.0 ** 24
    x[1:8, 0] = 1.0
    assert orc.column_sums_f32_ordered(x)[0] == np.float32(2.0 ** 24 + 4)
    assert orc.column_sums(x)[0] == 2.0 ** 24 + 7
    # balanced tree over the eight row groups: g0 = 2^24, g1 = g2 = g3 = 1 (one row each)
    # -> (2^24 + 1) + (1 + 1) = 2^24 + 2, where a left-to-right chain would lose all three ones
    x = np.zeros((32, 1), np.float32)
    x[0, 0], x[4, 0], x[8, 0], x[12, 0] = 2.0 ** 24, 1.0, 1.0, 1.0
    assert orc.column_sums_f32_ordered(x)[0] == np.float32(2.0 ** 24 + 2)
    # blocks: 9 blocks make runs of 2.  Block 0 = 2^24 and blocks 2, 3 = 1: run 1 = 1 + 1 = 2 survives,
    # 2^24 + 2 (one chain over the blocks in index order would lose both ones).  Block 0 = 2^24 and
    # blocks 1, 2 = 1: block 1 is lost inside run 0 and run 1 = 1 is lost in the last chain: 2^24, where
    # the exact sum 2^24 + 2 is representable.
    x = np.zeros((9 * 256, 1), np.float32)
    x[0, 0], x[2 * 256, 0], x[3 * 256, 0] = 2.0 ** 24, 1.0, 1.0
    assert orc.column_sums_f32_ordered(x)[0] == np.float32(2.0 ** 24 + 2)
    x = np.zeros((9 * 256, 1), np.float32)
    x[0, 0], x[1 * 256, 0], x[2 * 256, 0] = 2.0 ** 24, 1.0, 1.0
    assert orc.column_sums_f32_ordered(x)[0] == np.float32(2.0 ** 24)
    assert orc.column_sums(x)[0] == 2.0 ** 24 + 2


# ------------------------------------------------- E3M0 elements (Table 7's format ablation) ----

E3M0_GRID = [0.0, 0.25, 0.5, 1.0, 2.0, 4.0, 8.0, 16.0]


def test_e3m0_table_from_bit_fields(orc):
    """sign | 3 exponent bits | no mantissa bit, bias 3: exponent field 0 is the (empty) subnormal range,
    i.e. 0; field E >= 1 is 2^(E - 3).  Largest value 16 = 2^4: Q_p = 16, E_max = 4."""
    for code in range(16):
        E, sign = code & 7, code >> 3
        mag = 0.0 if E == 0 else 2.0 ** (E - 3)
        v = orc.e3m0_value(code)
        assert abs(v) == mag and (math.copysign(1.0, v) < 0) == bool(sign)
    assert max(orc.e3m0_value(c) for c in range(16)) == 16.0
    assert sorted(abs(orc.e3m0_value(c)) for c in range(8)) == E3M0_GRID


def test_e3m0_shared_exponent_vs_exact_rational(orc):
    """Sec. 3.2's two rules with Q_p - Q_n = 32 and E_max = 4 against exact rational arithmetic, incl.
    exact powers of two (the only values where the ceiling does not round up) and their neighbours."""
    rng = np.random.default_rng(21)
    bits = rng.integers(0x00800000, 0x7F000000, size=3000, dtype=np.uint32)
    special = [((e + 127) << 23) | m for e in range(-120, 120, 7) for m in (0, 1, 0x400000, 0x7FFFFF)]
    bits = np.concatenate([bits, np.array(special, np.uint32)])
    for u, v in zip(bits.tolist(), bits.view(np.float32).tolist()):
        fr = Fraction(v)
        tf = _exact_ceil_log2(2 * fr / 32)
        fl = _exact_floor_log2(fr) - 4
        assert orc.shared_exponent_e3m0(v, orc.SCALE_TRUNCFREE) == max(-127, min(127, tf))
        assert orc.shared_exponent_e3m0(v, orc.SCALE_FLOOR) == max(-127, min(127, fl))
        e, m = (u >> 23) - 127, u & 0x7FFFFF
        assert tf == e - 4 + (1 if m > 0 else 0) and fl == e - 4
    # the worked magnitude of Sec. 3.2, M = 31: truncation-free S = 2 (15.5 fits), Eq. 2's S = 1 (31 is cut to 16)
    assert orc.shared_exponent_e3m0(31.0, orc.SCALE_TRUNCFREE) == 1
    assert orc.shared_exponent_e3m0(31.0, orc.SCALE_FLOOR) == 0
    # all-zero group: epsilon = 1e-8
    eps = PAPER["zero_group_epsilon"]["epsilon"]
    assert orc.shared_exponent_e3m0(0.0, orc.SCALE_TRUNCFREE) == math.ceil(math.log2(eps / 16)) == -30
    assert orc.shared_exponent_e3m0(0.0, orc.SCALE_FLOOR) == math.floor(math.log2(eps)) - 4 == -31
    assert orc.shared_exponent_e3m0(float(np.float32(1e-45)), orc.SCALE_TRUNCFREE) == -127


def test_e3m0_rtn_brute_force_and_ties(orc):
    """Every bf16 value in [-16, 16]: the nearest of the 15 values, a midpoint to the larger value."""
    signed = sorted(set([-g for g in E3M0_GRID] + E3M0_GRID))
    grid = np.array(signed)
    u = np.arange(65536, dtype=np.uint32) << 16
    y = u.view(np.float32)
    y = y[np.isfinite(y) & (np.abs(y) <= 16.0)]
    for v in y.tolist():
        d = np.abs(grid - v)
        best = grid[np.flatnonzero(d == d.min()).max()]
        code = orc.round_rtn_e3m0(v)
        assert orc.e3m0_value(code) == best, v
        assert (code >> 3) == (1 if math.copysign(1.0, v) < 0 else 0)
    ties = {0.125: 0.25, 0.375: 0.5, 0.75: 1.0, 1.5: 2.0, 3.0: 4.0, 6.0: 8.0, 12.0: 16.0,
            -0.125: 0.0, -0.375: -0.25, -0.75: -0.5, -1.5: -1.0, -3.0: -2.0, -6.0: -4.0, -12.0: -8.0}
    for yv, want in ties.items():
        assert orc.e3m0_value(orc.round_rtn_e3m0(yv)) == want


def test_e3m0_sr_exhaustive_counts(orc):
    for y in (0.1, 0.125, 0.3, 1.2, 1.999, 2.75, 5.0, 11.0, 15.999, -0.3, -2.2, -9.0, 1e-6, 4.0, -16.0, 0.0):
        y = f32(y)
        a = abs(y)
        m1 = max(g for g in E3M0_GRID if g <= a)
        m2 = min([g for g in E3M0_GRID if g > m1] or [m1])
        p = (Fraction(a) - Fraction(m1)) / Fraction(m2 - m1) if m2 > m1 else Fraction(0)
        ups = 0
        for r in range(0, 65536):
            v = orc.e3m0_value(orc.round_sr_e3m0(y, r))
            assert abs(v) in (m1, m2) and (v == 0 or (v < 0) == (y < 0))
            ups += abs(v) == m2 and m2 > m1
        assert ups == math.ceil(65536 * p), y


def test_e3m0_quantize_invariants(orc):
    """Range invariants of the two scale rules, the error bound of round_D (half the gap of the cell the
    scaled value lies in), 2^k equivariance, Eq. 2's rule always putting the group maximum on +-16, the
    all-zero group, the pack layout, and stochastic decisions recomposed from (sr_bits, round_sr)."""
    rng = np.random.default_rng(22)
    x = (rng.standard_normal((48, 160)) * np.exp(rng.uniform(-15, 15, (48, 1)))).astype(np.float32)
    x[5, 32:64] = 0.0
    M = np.abs(x.reshape(48, 5, 32)).max(-1).astype(np.float64)
    nz = M > 0
    c, s = orc.quantize_e3m0(x, scale_mode=orc.SCALE_TRUNCFREE)
    S = 2.0 ** (s.astype(np.int64) - 127)
    r = M / S
    assert np.all(r[nz] <= 16.0) and np.all(r[nz] > 8.0)
    assert s[5, 1] == 127 - 30 and np.all(c[5, 16:32] == 0)
    d = orc.dequantize_e3m0(c, s)
    y = np.abs(x.astype(np.float64)) / np.repeat(S, 32, axis=1)
    lo = np.where(y >= 0.25, 2.0 ** np.floor(np.log2(np.maximum(y, 1e-300))), 0.0)
    gap = np.where(y >= 0.25, lo, 0.25)
    assert np.all(np.abs(np.abs(d) - np.abs(x.astype(np.float64))) <= 0.5 * gap * np.repeat(S, 32, axis=1) + 1e-300)
    c8, s8 = orc.quantize_e3m0(x * np.float32(8.0), scale_mode=orc.SCALE_TRUNCFREE)
    assert np.array_equal(c8, c) and np.array_equal(s8.astype(np.int64)[nz], s.astype(np.int64)[nz] + 3)
    cf, sf = orc.quantize_e3m0(x, scale_mode=orc.SCALE_FLOOR)
    rf = M / 2.0 ** (sf.astype(np.int64) - 127)
    assert np.all(rf[nz] >= 16.0) and np.all(rf[nz] < 32.0)
    df = np.abs(orc.dequantize_e3m0(cf, sf)).reshape(48, 5, 32).max(-1)
    assert np.all(df[nz] == 16.0 * 2.0 ** (sf.astype(np.int64) - 127)[nz])
    assert sf[5, 1] == 127 - 31
    # pack layout: low nibble = even column
    codes = [orc.round_rtn_e3m0(float(np.float32(v)) / float(S[0, 0])) for v in x[0, :4]]
    assert c[0, 0] == codes[0] | (codes[1] << 4) and c[0, 1] == codes[2] | (codes[3] << 4)
    # stochastic rounding follows the element index of the source
    cs, ss = orc.quantize_e3m0(x, round=orc.ROUND_SR, seed=77, tensor_id=3, index_base=1 << 33)
    assert np.array_equal(ss, s)
    for (rr, cc) in ((0, 0), (7, 33), (47, 159), (20, 100)):
        e = (1 << 33) + rr * 160 + cc
        yv = float(np.float32(x[rr, cc])) / float(S[rr, cc // 32])
        want = orc.round_sr_e3m0(np.float32(yv), orc.sr_bits(77, 3, e)) if abs(yv) >= 2.0 ** -100 else None
        got = (cs[rr, cc // 2] >> (4 * (cc & 1))) & 15
        if want is not None:
            assert got == want


# ------------------------------------------------- GELU (between the MLP's two linear layers) ----

def test_gelu_against_library_routines_and_identities(orc):
    """x * Phi(x): against scipy's normal distribution function and torch's FP64 GELU, the textbook
    values at 0 and +-1, the identity GELU(x) - GELU(-x) = x (Phi(x) + Phi(-x) = 1), GELU(x) -> x for
    large x, a correctly signed and relatively accurate negative tail (x Phi(x) with Phi from its
    asymptotic series), and |GELU'| <= 1.13 (the Lipschitz constant the fused kernel's tolerance uses)."""
    import torch
    from scipy.special import ndtr
    x = np.concatenate([np.linspace(-12, 12, 4001), np.array([0.0, -0.0, 1e-300, -1e-300, 1.0, -1.0, 37.0, -37.0])])
    g = orc.gelu(x)
    assert np.allclose(g, x * ndtr(x), rtol=1e-12, atol=0)       # two libm implementations of erfc
    # torch forms 1 + erf(x / sqrt 2), which cancels in the negative tail: compared where that is harmless
    mid = np.abs(x) <= 5
    assert np.allclose(g[mid], torch.nn.functional.gelu(torch.from_numpy(x[mid])).numpy(), rtol=1e-9, atol=1e-15)
    assert orc.gelu([0.0])[0] == 0.0
    assert abs(orc.gelu([1.0])[0] - 0.8413447460685429) < 1e-15
    assert abs(orc.gelu([-1.0])[0] + 0.15865525393145707) < 1e-15
    assert np.allclose(orc.gelu(x) - orc.gelu(-x), x, rtol=0, atol=1e-14)
    assert orc.gelu([40.0])[0] == 40.0
    t = -9.0                                            # Phi(t) ~ phi(t)/|t| * (1 - 1/t^2 + 3/t^4 - 15/t^6)
    phi = math.exp(-t * t / 2) / math.sqrt(2 * math.pi)
    series = phi / abs(t) * (1 - 1 / t ** 2 + 3 / t ** 4 - 15 / t ** 6)
    assert abs(orc.gelu([t])[0] / (t * series) - 1) < 1e-5 and orc.gelu([t])[0] < 0
    xs = np.linspace(-8, 8, 200001)
    slope = np.diff(orc.gelu(xs)) / np.diff(xs)
    assert slope.max() < 1.13 and slope.min() > -0.13


def test_fused_reference_is_the_composition(orc):
    """linear_fwd_gelu_quant = product + bias, GELU, row quantizer, on a tiny layer by hand."""
    rng = np.random.default_rng(31)
    X = rng.standard_normal((4, 64)).astype(np.float32)
    W = (rng.standard_normal((32, 64)) * 0.3).astype(np.float32)
    bias = rng.standard_normal(32).astype(np.float32)
    xq, xs = orc.quantize(X)
    wq, ws = orc.quantize(W)
    P, A, c, s = orc.linear_fwd_gelu_quant(xq, xs, wq, ws, bias)
    Pn = orc.dequantize(xq, xs) @ orc.dequantize(wq, ws).T + bias.astype(np.float64)
    assert np.allclose(P, Pn, rtol=1e-14, atol=1e-14)
    from scipy.special import ndtr
    assert np.allclose(A, Pn * ndtr(Pn), rtol=1e-12, atol=1e-300)
    c2, s2 = orc.quantize(A.astype(np.float32))
    assert np.array_equal(c, c2) and np.array_equal(s, s2)
