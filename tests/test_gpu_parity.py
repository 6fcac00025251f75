"""Parity of the HIP path (through the C ABI) with the CPU oracle on the same
seeded inputs.  Codes, scale bytes and rounding decisions must match bit for bit;
products must agree with the FP64 product of the same dequantized operands to
1e-5 (normwise, and per entry relative to sum_k |a||b|)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def mx():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2502_20853_amd as mx
    mx.binding.lib()
    return mx


def dev(a, dtype="f32"):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def assert_same_bytes(got, want, what):
    got = host(got)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    bad = np.flatnonzero(got.ravel() != want.ravel())
    assert bad.size == 0, "%s: %d of %d bytes differ, first at %d (got %d want %d)" % (
        what, bad.size, want.size, bad[0], got.ravel()[bad[0]], want.ravel()[bad[0]])


def mixed_matrix(rows, cols, seed, dtype):
    import mx_workloads as wl
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, cols)).astype(np.float32)
    x *= np.exp(rng.uniform(-6, 6, (rows, 1))).astype(np.float32)     # row scales spread over many binades
    x[:, rng.integers(0, cols, 3)] *= 20
    x[rng.integers(0, rows, 4), :32] = 0                              # all-zero groups
    x[0, :8] = [0.25, 0.75, -0.25, -0.75, 2.5, -2.5, 5.0, -5.0]       # exact midpoints after scaling
    x[0, 8] = 6.0
    if rows > 1:
        x[1, :4] = [-0.0, 0.0, 1e-30, -1e-30]
    return wl.round_to_bf16(x) if dtype == "bf16" else x


# ------------------------------------------------------------------ rows ----

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rnd", [0, 1])
@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("shape", [(256, 192), (37, 1056), (1, 32)])
def test_quantize_rows(mx, orc, dtype, rnd, mode, shape):
    x = mixed_matrix(*shape, seed=10 + shape[0], dtype=dtype)
    want = orc.quantize(x, round=rnd, scale_mode=mode, seed=77, tensor_id=3, index_base=4096)
    got = mx.mx_quantize(dev(x, dtype), rnd, mode, seed=77, tensor_id=3, index_base=4096)
    assert_same_bytes(got[1], want[1], "scales")
    assert_same_bytes(got[0], want[0], "codes")


def test_quantize_rows_strided_and_seed_64bit(mx, orc):
    big = mixed_matrix(64, 256, seed=3, dtype="bf16")
    view = big[:, 64:192]
    seed = 0xDEADBEEF12345678
    want = orc.quantize(view, round=1, seed=seed, tensor_id=0xFFFFFFFF, index_base=(1 << 36) + 8)
    t = dev(big, "bf16")[:, 64:192]
    got = mx.mx_quantize(t, 1, 0, seed=seed, tensor_id=0xFFFFFFFF, index_base=(1 << 36) + 8)
    assert_same_bytes(got[0], want[0], "codes")
    assert_same_bytes(got[1], want[1], "scales")


def test_quantize_extreme_values(mx, orc):
    # subnormals, the clamp at s = -127, the largest finite inputs, exact powers of two and 1.5*2^e
    rows = 64
    x = np.zeros((rows, 64), np.float32)
    bits = np.array([0x00000001, 0x00000100, 0x007FFFFF, 0x00800000, 0x00C00000, 0x00C00001, 0x01000000,
                     0x3FC00000, 0x3FC00001, 0x3FBFFFFF, 0x7F7FFFFF, 0x7F000000, 0x7E800000, 0x40C00000,
                     0x40C00001, 0x3F800000], np.uint32)
    for i, b in enumerate(bits):
        x[i, 0] = np.array([b], np.uint32).view(np.float32)[0]
        x[i, 1:32] = x[i, 0] * np.linspace(-1, 1, 31, dtype=np.float32)
        x[i, 32] = -x[i, 0]
        x[i, 33:64] = x[i, 0] * np.float32(2.0) ** -np.arange(1, 32, dtype=np.float32) * 1.7
    rng = np.random.default_rng(0)
    x[16:] = rng.standard_normal((rows - 16, 64)).astype(np.float32) * np.float32(2.0) ** rng.integers(-140, 120, (rows - 16, 1)).astype(np.float32)
    x = np.nan_to_num(x, posinf=3e38, neginf=-3e38)
    for rnd in (0, 1):
        for mode in (0, 1):
            want = orc.quantize(x, round=rnd, scale_mode=mode, seed=5, tensor_id=1)
            got = mx.mx_quantize(dev(x), rnd, mode, seed=5, tensor_id=1)
            assert_same_bytes(got[1], want[1], "scales r%d m%d" % (rnd, mode))
            assert_same_bytes(got[0], want[0], "codes r%d m%d" % (rnd, mode))


def test_sr_zero_draw_on_tiny_elements(mx, orc):
    # elements whose 16 random bits are 0 round up iff p > 0, however small p is:
    # put values ~2^-40 of the group maximum exactly there
    seed, tid, n = 9, 2, 1 << 18
    r = np.array([orc.sr_bits(seed, tid, e) for e in range(n)])
    zeros = np.flatnonzero(r == 0)
    assert zeros.size > 0
    x = np.ones(n, np.float32)
    x[zeros] = np.float32(2.0) ** -40
    x[zeros[::2]] = np.float32(2.0) ** -140          # scaled value underflows to a subnormal
    x = x.reshape(-1, 256)
    want = orc.quantize(x, round=1, seed=seed, tensor_id=tid)
    got = mx.mx_quantize(dev(x), 1, 0, seed=seed, tensor_id=tid)
    assert_same_bytes(got[0], want[0], "codes")
    flat = orc.dequantize(*want).ravel()
    assert np.all(flat[zeros] > 0)                   # they did round up to 0.5 * S


def test_tiny_elements_under_a_large_scale(mx, orc):
    # quotients far below FP32's range: every rounding rule must still see them as nonzero
    rng = np.random.default_rng(8)
    x = np.zeros((64, 128), np.float32)
    x[:, ::32] = np.float32(2.0) ** rng.integers(0, 60, (64, 4)).astype(np.float32)       # group maxima
    tiny = np.float32(2.0) ** rng.integers(-149, -100, (64, 128)).astype(np.float32)
    tiny *= rng.choice(np.array([-1.0, 1.0], np.float32), (64, 128))
    mask = np.ones_like(x, bool)
    mask[:, ::32] = False
    x[mask] = tiny[mask]
    for rnd in (0, 1):
        for seed in range(3):
            want = orc.quantize(x, round=rnd, seed=seed, tensor_id=1)
            got = mx.mx_quantize(dev(x), rnd, 0, seed=seed, tensor_id=1)
            assert_same_bytes(got[0], want[0], "codes r%d" % rnd)
        kw = dict(round_t=rnd, tensor_id_t=2, pre_quant=0, want_row=True, round_row=1 - rnd, tensor_id_row=3, seed=5)
        want = orc.quantize_transposed(x, **kw)
        got = mx.mx_quantize_transposed(dev(x), **kw)
        for i, nm in enumerate(["codes_t", "scales_t", "codes_row", "scales_row"]):
            assert_same_bytes(got[i], want[i], nm)
    ema = np.abs(x) * np.float32(2.0) ** 40
    ema = np.minimum(ema, np.float32(1e30)).astype(np.float32)
    want = orc.ema_weight_quant(x, ema.copy(), update_ema=0)
    got = mx.mx_ema_weight_quant(dev(x), dev(ema), 0.5, 0)
    assert_same_bytes(got[0], want[0], "ema codes")


# ------------------------------------------------------------ transposed ----

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("pre,rr,rt,want_row", [(1, 0, 1, True), (0, 1, 1, True), (1, 0, 0, False),
                                                 (0, 0, 1, False), (1, 1, 1, True), (0, 0, 0, True)])
@pytest.mark.parametrize("shape", [(256, 192), (96, 320), (32, 32), (544, 96)])
def test_quantize_transposed(mx, orc, dtype, pre, rr, rt, want_row, shape):
    x = mixed_matrix(*shape, seed=20 + shape[1], dtype=dtype)
    kw = dict(round_t=rt, tensor_id_t=6, pre_quant=pre, want_row=want_row, round_row=rr, tensor_id_row=1,
              seed=1234, index_base=64)
    want = orc.quantize_transposed(x, **kw)
    got = mx.mx_quantize_transposed(dev(x, dtype), **kw)
    names = ["codes_t", "scales_t", "codes_row", "scales_row"]
    for i in (1, 0, 3, 2):
        if want[i] is None:
            assert got[i] is None
        else:
            assert_same_bytes(got[i], want[i], names[i])


@pytest.mark.parametrize("mode", [0, 1])
def test_quantize_transposed_floor_and_given_row(mx, orc, mode):
    x = mixed_matrix(128, 160, seed=31, dtype="bf16")
    kw = dict(round_t=1, tensor_id_t=4, pre_quant=1, want_row=True, round_row=0, tensor_id_row=2,
              scale_mode=mode, seed=99)
    want = orc.quantize_transposed(x, **kw)
    got = mx.mx_quantize_transposed(dev(x, "bf16"), **kw)
    for i, nm in enumerate(["codes_t", "scales_t", "codes_row", "scales_row"]):
        assert_same_bytes(got[i], want[i], nm)
    # same result when the row codes are handed in and no source is given
    rc, rs = dev(want[2]), dev(want[3])
    got2 = mx.mx_quantize_transposed(None, 1, 4, 1, False, row_in=(rc, rs), scale_mode=mode, seed=99,
                                     shape=x.shape)
    assert_same_bytes(got2[0], want[0], "codes_t (given row)")
    assert_same_bytes(got2[1], want[1], "scales_t (given row)")


def test_quantize_transposed_strided(mx, orc):
    big = mixed_matrix(64, 384, seed=41, dtype="f32")
    kw = dict(round_t=1, tensor_id_t=5, pre_quant=0, want_row=True, round_row=1, tensor_id_row=3, seed=7)
    want = orc.quantize_transposed(big[:, 128:352], **kw)
    got = mx.mx_quantize_transposed(dev(big)[:, 128:352], **kw)
    for i, nm in enumerate(["codes_t", "scales_t", "codes_row", "scales_row"]):
        assert_same_bytes(got[i], want[i], nm)


# ----------------------------------------------------------------- Q-EMA ----

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode", [0, 1])
def test_ema_weight_quant(mx, orc, dtype, mode):
    import mx_workloads as wl
    steps = list(wl.weight_walk(96, 160, seed=0, steps=6, sigma=4e-4))
    ema_o = np.zeros_like(steps[0])
    ema_g = torch.zeros(steps[0].shape, dtype=torch.float32, device="cuda")
    for t, w in enumerate(steps):
        w = wl.round_to_bf16(w) if dtype == "bf16" else w
        upd = 2 if t == 0 else 1
        want = orc.ema_weight_quant(w, ema_o, beta=0.9, update_ema=upd, scale_mode=mode)
        got = mx.mx_ema_weight_quant(dev(w, dtype), ema_g, 0.9, upd, mode)
        assert_same_bytes(ema_g.view(torch.uint8), ema_o.view(np.uint8), "w_ema step %d" % t)
        assert_same_bytes(got[1], want[1], "scales step %d" % t)
        assert_same_bytes(got[0], want[0], "codes step %d" % t)
    # update_ema = 0 leaves the state alone; an EMA far from w still stays inside w's bracket
    before = host(ema_g).copy()
    far = (steps[-1] * np.float32(-3.0)).astype(np.float32)
    want = orc.ema_weight_quant(steps[-1], far.copy(), update_ema=0, scale_mode=mode)
    got = mx.mx_ema_weight_quant(dev(steps[-1]), dev(far), 0.5, 0, mode)
    assert_same_bytes(got[0], want[0], "codes far ema")
    assert np.array_equal(host(ema_g), before)


# ------------------------------------------------------------------ GEMM ----

def random_packed(rows, k, seed, scale_lo=110, scale_hi=140):
    rng = np.random.default_rng(seed)
    codes = rng.integers(0, 256, (rows, k // 2), dtype=np.uint8)
    scales = rng.integers(scale_lo, scale_hi, (rows, k // 32), dtype=np.uint8)
    return codes, scales


def check_product(orc, got, ac, as_, bc, bs, what, tol=1e-5):
    ref = orc.gemm_f64(ac, as_, bc, bs)
    absref = np.abs(orc.dequantize(ac, as_)) @ np.abs(orc.dequantize(bc, bs)).T
    got = host(got).astype(np.float64)
    assert got.shape == ref.shape
    err = np.abs(got - ref)
    assert np.linalg.norm(err) <= tol * np.linalg.norm(ref), (what, np.linalg.norm(err) / np.linalg.norm(ref))
    worst = (err / (absref + 1e-300)).max()
    assert worst <= tol, (what, worst)


@pytest.mark.parametrize("m,n,k", [(256, 768, 192), (16, 16, 128), (1, 1, 32), (300, 200, 96),
                                    (515, 260, 1056), (64, 1000, 4096), (257, 255, 160),
                                    # K % 128 == 0: the DMA-fed 32x32x64 kernel (1 to 11 K steps, ragged m and n)
                                    (1, 1, 128), (256, 256, 128), (300, 200, 384), (515, 260, 1024),
                                    (257, 129, 256), (33, 700, 1408), (768, 768, 512),
                                    # >= 4 K steps: 256-K stages, odd step counts, shifted last scale block
                                    (40, 48, 640), (300, 520, 1152), (130, 260, 896), (64, 64, 2688),
                                    # K splits of unequal length (10,10,10,7 steps) and a last split too short
                                    # for the main kernel (9 x 6 + 3 steps: the short-K kernel takes it all)
                                    (100, 300, 4736), (70, 130, 7296)])
def test_gemm_random_codes(mx, orc, m, n, k):
    ac, as_ = random_packed(m, k, 1)
    bc, bs = random_packed(n, k, 2)
    got = mx.mx_linear_fwd(dev(ac), dev(as_), dev(bc), dev(bs))
    check_product(orc, got, ac, as_, bc, bs, "fwd %dx%dx%d" % (m, n, k))


@pytest.mark.parametrize("m,n,k", [(6100, 2900, 640), (9000, 2500, 896), (4200, 4000, 512)])
def test_gemm_more_tiles_than_resident_workgroups(mx, orc, m, n, k):
    # over 512 output tiles: workgroups of the persistent kernel walk several tiles, with odd and even
    # K step counts (the stage-buffer parity carries over from tile to tile) and ragged edge tiles
    ac, as_ = random_packed(m, k, 21, 120, 134)
    bc, bs = random_packed(n, k, 22, 120, 134)
    got = host(mx.mx_linear_fwd(dev(ac), dev(as_), dev(bc), dev(bs))).astype(np.float64)
    rng = np.random.default_rng(k)
    ii = np.concatenate([rng.integers(0, m, 20000), [0, m - 1, 0, m - 1]])
    jj = np.concatenate([rng.integers(0, n, 20000), [0, 0, n - 1, n - 1]])
    ref, absref = orc.gemm_f64_sampled(ac, as_, bc, bs, ii, jj)
    assert np.all(np.abs(got[ii, jj] - ref) <= 1e-5 * absref)
    # every tile is covered: row and column sums of the full product against FP64 sums
    A, B = orc.dequantize(ac, as_), orc.dequantize(bc, bs)
    col = A.sum(axis=0) @ B.T
    colabs = np.abs(A).sum(axis=0) @ np.abs(B).T
    assert np.all(np.abs(got.sum(axis=0) - col) <= 1e-5 * colabs)
    row = A @ B.sum(axis=0)
    rowabs = np.abs(A) @ np.abs(B).sum(axis=0)
    assert np.all(np.abs(got.sum(axis=1) - row) <= 1e-5 * rowabs)


@pytest.mark.parametrize("out", ["f32", "bf16"])
@pytest.mark.parametrize("m,n,k", [(256, 768, 192), (300, 200, 96),             # 16x16x128 kernel, ragged tiles
                                    (300, 200, 384), (33, 700, 256),             # short-K 32x32x64 kernel
                                    (515, 260, 1024), (768, 768, 512), (40, 48, 640),   # main kernel; 4 columns in the last tile
                                    (64, 1000, 4096), (100, 300, 4736)])         # K split: the reduction adds the bias
def test_linear_fwd_bias(mx, orc, m, n, k, out):
    """Y = A.B^T + bias with the bias added before the one rounding to the output type, on every kernel
    path; against the FP64 product of the same operands plus the bias."""
    ac, as_ = random_packed(m, k, 31, 125, 129)
    bc, bs = random_packed(n, k, 32, 125, 129)
    bias = (np.random.default_rng(n).standard_normal(n) * 64).astype(np.float32)
    bias[: min(4, n)] = [0.0, -0.0, 1e-3, -4096.0][: min(4, n)]
    got = mx.mx_linear_fwd_bias(dev(ac), dev(as_), dev(bc), dev(bs), dev(bias),
                                out_dtype=torch.bfloat16 if out == "bf16" else torch.float32)
    ref = orc.gemm_f64(ac, as_, bc, bs) + bias.astype(np.float64)[None, :]
    absref = np.abs(orc.dequantize(ac, as_)) @ np.abs(orc.dequantize(bc, bs)).T + np.abs(bias)[None, :]
    tol = 1e-5 * absref + (np.abs(ref) * 2.0 ** -8 if out == "bf16" else 0.0)
    err = np.abs(host(got.float()).astype(np.float64) - ref)
    assert np.all(err <= tol), (np.max(err / (absref + 1e-300)), np.unravel_index(np.argmax(err / (tol + 1e-300)), err.shape))


def test_linear_fwd_bias_strided_output_of_a_k_split(mx, orc):
    """K split whose output rows are not 16-byte aligned: the scalar form of the reduction adds the bias."""
    m, n, k = 64, 1000, 4096
    ac, as_ = random_packed(m, k, 33, 125, 129)
    bc, bs = random_packed(n, k, 34, 125, 129)
    bias = np.random.default_rng(5).standard_normal(n).astype(np.float32)
    wide = torch.zeros((m, n + 1), dtype=torch.float32, device="cuda")
    mx.mx_linear_fwd_bias(dev(ac), dev(as_), dev(bc), dev(bs), dev(bias), out=wide[:, :n])
    ref = orc.gemm_f64(ac, as_, bc, bs) + bias.astype(np.float64)[None, :]
    absref = np.abs(orc.dequantize(ac, as_)) @ np.abs(orc.dequantize(bc, bs)).T + np.abs(bias)[None, :]
    got = host(wide).astype(np.float64)
    assert np.all(np.abs(got[:, :n] - ref) <= 1e-5 * absref) and np.all(got[:, n] == 0)


@pytest.mark.parametrize("m,n,k", [(8192, 6400, 512), (6100, 2900, 640)])
def test_linear_fwd_bias_over_several_tiles_per_workgroup(mx, orc, m, n, k):
    """More output tiles than workgroups (up to 3.1 per workgroup at the shortest K loop the main kernel
    takes): each tile must see its own 256 bias values.  The bias encodes its column, so a value from
    another tile's slot is far outside the tolerance."""
    ac, as_ = random_packed(m, k, 35, 120, 130)
    bc, bs = random_packed(n, k, 36, 120, 130)
    bias = (np.arange(n, dtype=np.float32) - n / 2) * 4096.0
    got = host(mx.mx_linear_fwd_bias(dev(ac), dev(as_), dev(bc), dev(bs), dev(bias))).astype(np.float64)
    rng = np.random.default_rng(k)
    ii = np.concatenate([rng.integers(0, m, 30000), [0, m - 1, 0, m - 1]])
    jj = np.concatenate([rng.integers(0, n, 30000), [0, 0, n - 1, n - 1]])
    ref, absref = orc.gemm_f64_sampled(ac, as_, bc, bs, ii, jj)
    assert np.all(np.abs(got[ii, jj] - (ref + bias[jj])) <= 1e-5 * (absref + np.abs(bias[jj])))
    # every entry: subtracting the bias must leave the plain product
    plain = host(mx.mx_linear_fwd(dev(ac), dev(as_), dev(bc), dev(bs))).astype(np.float64)
    assert np.all(np.abs((got - bias[None, :]) - plain) <= 2.0 ** -22 * (np.abs(plain) + np.abs(bias)[None, :]) + 1e-30)


def test_gemm_scale_bytes_and_one_hot(mx, orc):
    # operand with a single nonzero per row pins the lane <-> (row, K block) mapping of codes and scales
    m, n, k = 48, 40, 256
    ac = np.zeros((m, k // 2), np.uint8)
    bc = np.full((n, k // 2), 0x22, np.uint8)                 # all ones (code 2 = 1.0)
    as_ = np.full((m, k // 32), 127, np.uint8)
    bs = np.zeros((n, k // 32), np.uint8)
    for j in range(n):
        bs[j] = 120 + (np.arange(k // 32) + j) % 16           # a different power of two per (row, group)
    for i in range(m):
        kk = (37 * i + 5) % k
        ac[i, kk // 2] = 0x05 if kk % 2 == 0 else 0x50        # 3.0 at column kk
        as_[i, kk // 32] = 127 + (i % 5)
    got = mx.mx_linear_fwd(dev(ac), dev(as_), dev(bc), dev(bs))
    ref = orc.gemm_f64(ac, as_, bc, bs)
    assert np.array_equal(host(got).astype(np.float64), ref)  # single products of powers of two: exact


def test_gemm_three_entry_points_and_split_k(mx, orc):
    N, C, D = 4096 + 32, 96, 160                              # dW contracts over N: K-split path
    xc, xs = random_packed(N, D, 3)
    wc, ws = random_packed(C, D, 4)
    dyc, dys = random_packed(N, C, 5, 100, 120)
    wtc, wts = random_packed(D, C, 6)
    dytc, dyts = random_packed(C, N, 7, 100, 120)
    xtc, xts = random_packed(D, N, 8)
    check_product(orc, mx.mx_linear_fwd(dev(xc), dev(xs), dev(wc), dev(ws)), xc, xs, wc, ws, "fwd")
    check_product(orc, mx.mx_linear_bwd_dx(dev(dyc), dev(dys), dev(wtc), dev(wts)), dyc, dys, wtc, wts, "dx")
    assert mx.mx_linear_workspace_bytes(mx.GEMM_BWD_DW, N, C, D) > 0
    check_product(orc, mx.mx_linear_bwd_dw(dev(dytc), dev(dyts), dev(xtc), dev(xts)), dytc, dyts, xtc, xts, "dw")


@pytest.mark.parametrize("m,n,k", [(130, 72, 224), (130, 72, 256), (300, 263, 384)])
def test_gemm_bf16_output_and_ld(mx, orc, m, n, k):
    ac, as_ = random_packed(m, k, 11, 120, 130)
    bc, bs = random_packed(n, k, 12, 120, 130)
    ref = orc.gemm_f64(ac, as_, bc, bs)
    out = torch.full((m, n + 8), 7.0, dtype=torch.bfloat16, device="cuda")
    mx.mx_linear_fwd(dev(ac), dev(as_), dev(bc), dev(bs), out=out[:, :n])
    got = host(out.float())
    assert np.all(got[:, n:] == 7.0)                          # columns beyond n untouched
    absref = np.abs(orc.dequantize(ac, as_)) @ np.abs(orc.dequantize(bc, bs)).T
    assert np.all(np.abs(got[:, :n] - ref) <= np.abs(ref) * 2.0 ** -8 + 1e-5 * absref)   # one bf16 ulp
    f32 = host(mx.mx_linear_fwd(dev(ac), dev(as_), dev(bc), dev(bs)))
    want = host(torch.from_numpy(f32).cuda().to(torch.bfloat16).float())
    assert np.array_equal(got[:, :n], want)                   # RNE of the FP32 result


# ------------------------------------------------------------ whole layer ----

def oracle_layer(orc, X, W, dY, seed):
    xt = orc.quantize_transposed(X, round_t=1, tensor_id_t=6, pre_quant=1, round_row=0, tensor_id_row=1, seed=seed)
    wt = orc.quantize_transposed(W, round_t=1, tensor_id_t=4, pre_quant=1, round_row=0, tensor_id_row=2, seed=seed)
    dy = orc.quantize_transposed(dY, round_t=1, tensor_id_t=5, pre_quant=0, round_row=1, tensor_id_row=3, seed=seed)
    return xt, wt, dy


def test_layer_c1_single(mx, orc):
    import mx_workloads as wl
    N, D, C = 256, 192, 768
    X, W, dY = wl.linear_layer(N, D, C, seed=0, dtype="f32", outliers=4)
    xt, wt, dy = oracle_layer(orc, X, W, dY, seed=0)
    step = mx.MxLinearStep(N, D, C, out_dtype=torch.float32)
    y = step.forward(dev(X), dev(W), seed=0)
    dx, dw = step.backward(dev(dY), seed=0)
    for got, want, nm in ((step.xq, xt[2], "Q1"), (step.xs, xt[3], "S1"), (step.xtq, xt[0], "Q6"), (step.xts, xt[1], "S6"),
                          (step.wq, wt[2], "Q2"), (step.ws, wt[3], "S2"), (step.wtq, wt[0], "Q4"), (step.wts, wt[1], "S4"),
                          (step.dyq, dy[2], "Q3"), (step.dys, dy[3], "S3"), (step.dytq, dy[0], "Q5"), (step.dyts, dy[1], "S5")):
        assert_same_bytes(got, want, nm)
    check_product(orc, y, xt[2], xt[3], wt[2], wt[3], "Y")
    check_product(orc, dx, dy[2], dy[3], wt[0], wt[1], "dX")
    check_product(orc, dw, dy[0], dy[1], xt[0], xt[1], "dW")


def test_layer_qema_variant(mx, orc):
    import mx_workloads as wl
    N, D, C = 128, 96, 160
    X, _, dY = wl.linear_layer(N, D, C, seed=1)
    step = mx.MxLinearStep(N, D, C, out_dtype=torch.float32, qema=True, beta=0.998)
    ema = None
    for t, W in enumerate(wl.weight_walk(C, D, seed=1, steps=3)):
        if ema is None:
            ema = np.zeros_like(W)
        wc, wsc = orc.ema_weight_quant(W, ema, beta=0.998, update_ema=2 if t == 0 else 1)
        wt = orc.quantize_transposed(W, round_t=1, tensor_id_t=4, pre_quant=1, want_row=False, row_in=(wc, wsc), seed=t)
        y = step.forward(dev(X), dev(W), seed=t)
        assert_same_bytes(step.wq, wc, "Q-EMA codes step %d" % t)
        assert_same_bytes(step.wtq, wt[0], "Q4 of Q-EMA step %d" % t)
        assert_same_bytes(step.wts, wt[1], "S4 of Q-EMA step %d" % t)
    xq = orc.quantize(X)
    check_product(orc, y, xq[0], xq[1], wc, wsc, "Y with Q-EMA weight")


def test_determinism(mx):
    x = dev(mixed_matrix(256, 512, seed=5, dtype="bf16"), "bf16")
    a = mx.mx_quantize_transposed(x, 1, 6, 1, True, 0, 1, seed=3)
    b = mx.mx_quantize_transposed(x, 1, 6, 1, True, 0, 1, seed=3)
    c = mx.mx_quantize_transposed(x, 1, 6, 1, True, 0, 1, seed=4)
    assert all(torch.equal(p, q) for p, q in zip(a, b))
    assert torch.equal(a[2], c[2]) and not torch.equal(a[0], c[0])   # RTN row codes ignore the seed


# ------------------------------------------------- the other workload configurations ----

def _check_layer(mx, orc, step, xt, wt, dy, y, dx, dw, N, D, C, bf16_out, sampled_only, tag):
    for got, want, nm in ((step.xq, xt[2], "Q1"), (step.xs, xt[3], "S1"), (step.xtq, xt[0], "Q6"), (step.xts, xt[1], "S6"),
                          (step.wq, wt[2], "Q2"), (step.ws, wt[3], "S2"), (step.wtq, wt[0], "Q4"), (step.wts, wt[1], "S4"),
                          (step.dyq, dy[2], "Q3"), (step.dys, dy[3], "S3"), (step.dytq, dy[0], "Q5"), (step.dyts, dy[1], "S5")):
        if want is not None:
            assert_same_bytes(got, want, "%s %s" % (tag, nm))
    rng = np.random.default_rng(N + D + C)
    for out, ops, m, n, nm, bf in ((y, (xt[2], xt[3], wt[2], wt[3]), N, C, "Y", bf16_out),
                                   (dx, (dy[2], dy[3], wt[0], wt[1]), N, D, "dX", bf16_out),
                                   (dw, (dy[0], dy[1], xt[0], xt[1]), C, D, "dW", False)):
        if not sampled_only and not bf:
            check_product(orc, out, *ops, "%s %s" % (tag, nm))
            continue
        ii = rng.integers(0, m, 4096)
        jj = rng.integers(0, n, 4096)
        ii[:4], jj[:4] = [0, m - 1, 0, m - 1], [0, 0, n - 1, n - 1]
        ref, absref = orc.gemm_f64_sampled(*ops, ii, jj)
        got = host(out.float())[ii, jj].astype(np.float64)
        tol = 1e-5 * absref + (np.abs(ref) * 2.0 ** -8 if bf else 0.0)
        assert np.all(np.abs(got - ref) <= tol), (tag, nm, np.max(np.abs(got - ref) / (absref + 1e-300)))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_config_vit_tiny_all_layers(mx, orc, dtype):
    """ViT-Tiny batch 64 (N = 12608, not a multiple of 128): the four layers of a block, FP32 and bf16
    sources, FP32 outputs, every packed byte and every product entry checked."""
    import mx_workloads as wl
    for li, (name, N, D, C) in enumerate(wl.config_layers("vit_tiny_b64")):
        X, W, dY = wl.linear_layer(N, D, C, seed=li, dtype=dtype, outliers=4)
        step = mx.MxLinearStep(N, D, C, out_dtype=torch.float32)
        y = step.forward(dev(X, dtype), dev(W, dtype), seed=li)
        dx, dw = step.backward(dev(dY, dtype), seed=li)
        xt, wt, dy = oracle_layer(orc, X, W, dY, seed=li)
        _check_layer(mx, orc, step, xt, wt, dy, y, dx, dw, N, D, C, False, False, "vit_tiny %s %s" % (name, dtype))


def _config_layer(name, layer):
    import mx_workloads as wl
    for li, (ln, N, D, C) in enumerate(wl.config_layers(name)):
        if ln == layer:
            return li, N, D, C
    raise KeyError(layer)


@pytest.mark.parametrize("layer", ["qkv", "proj", "fc1", "fc2"])
def test_config_vit_small_layer(mx, orc, layer):
    """ViT-Small batch 128 (N = 25216 = 98.5 x 256), every layer of the block at full size, bf16 sources
    and outputs, stochastic rounding on all backward quantizers: all packed bytes, 4096 sampled entries
    of each product."""
    import mx_workloads as wl
    li, N, D, C = _config_layer("vit_small_b128", layer)
    X, W, dY = wl.linear_layer(N, D, C, seed=10 + li, dtype="bf16")
    step = mx.MxLinearStep(N, D, C, out_dtype=torch.bfloat16, dw_dtype=torch.float32)
    y = step.forward(dev(X, "bf16"), dev(W, "bf16"), seed=li)
    dx, dw = step.backward(dev(dY, "bf16"), seed=li)
    xt, wt, dy = oracle_layer(orc, X, W, dY, seed=li)
    _check_layer(mx, orc, step, xt, wt, dy, y, dx, dw, N, D, C, True, True, "vit_small " + layer)


@pytest.mark.parametrize("layer", ["qkv", "proj", "fc1", "fc2"])
def test_config_vit_large_qema_layer(mx, orc, layer):
    """ViT-Large batch 256, every layer of the block at full size with the weight through Q-EMA: 20 steps
    of the master-weight walk, each followed by the EMA update and quantization (codes and EMA state
    checked at every step); the last step's codes feed the forward product and, re-quantized by Q4, the
    dX product.  All packed bytes, 4096 sampled entries of each product."""
    import mx_workloads as wl
    li, N, D, C = _config_layer("vit_large_b256", layer)
    X, _, dY = wl.linear_layer(N, D, C, seed=5 + li, dtype="bf16")
    step = mx.MxLinearStep(N, D, C, out_dtype=torch.bfloat16, dw_dtype=torch.float32, qema=True, beta=0.998)
    ema = None
    for t, W in enumerate(wl.weight_walk(C, D, seed=5 + li, steps=20)):
        if ema is None:
            ema = np.zeros_like(W)
        wc, wsc = orc.ema_weight_quant(W, ema, beta=0.998, update_ema=2 if t == 0 else 1)
        step.quantize_weight(dev(W), seed=t)                  # EMA update + Q-EMA + Q4 of its result
        assert_same_bytes(step.wq, wc, "Q-EMA codes step %d" % t)
    assert np.array_equal(host(step.w_ema), ema)
    # X and the products with the step-20 weight (forward() would update the EMA once more)
    mx.mx_quantize_transposed(dev(X, "bf16"), 1, 6, 1, True, 0, 1, seed=20, out=(step.xtq, step.xts, step.xq, step.xs))
    y = mx.mx_linear_fwd(step.xq, step.xs, step.wq, step.ws, out=step.y, workspace=step.workspace)
    dx, dw = step.backward(dev(dY, "bf16"), seed=20)
    wt4 = orc.quantize_transposed(W, round_t=1, tensor_id_t=4, pre_quant=1, want_row=False, row_in=(wc, wsc), seed=20)
    xt = orc.quantize_transposed(X, round_t=1, tensor_id_t=6, pre_quant=1, round_row=0, tensor_id_row=1, seed=20)
    dy = orc.quantize_transposed(dY, round_t=1, tensor_id_t=5, pre_quant=0, round_row=1, tensor_id_row=3, seed=20)
    del X, dY
    wt = (wt4[0], wt4[1], wc, wsc)
    _check_layer(mx, orc, step, xt, wt, dy, y, dx, dw, N, D, C, True, True, "vit_large %s q-ema" % layer)


# ------------------------------------------------- column sums with the fused quantizer ----

@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("rows,cols", [(32, 32), (288, 320), (544, 96), (4096 + 96, 4096 + 160)])
def test_column_sums_with_the_fused_quantizer(mx, orc, dtype, rows, cols):
    """col_sums of the batched entry point: the sums of the source columns against FP64 (tolerance of an
    FP32 sum), bit-identical on a second call, and packed outputs unchanged by the option.  Shapes with
    ragged 256-row blocks, narrow tiles, and a wide launch with a narrow tail."""
    x = mixed_matrix(rows, cols + 8, seed=90 + rows, dtype=dtype)
    X = dev(x, dtype)[:, :cols]
    want = orc.quantize_transposed(np.ascontiguousarray(x[:, :cols]), round_t=1, tensor_id_t=5, pre_quant=0,
                                   round_row=1, tensor_id_row=3, seed=9)
    sums = []
    for rep in range(2):
        out = tuple(torch.empty(w.shape, dtype=torch.uint8, device="cuda") for w in want)
        cs = torch.full((cols,), float("nan"), device="cuda")
        mx.mx_quantize_transposed_batch([{"src": X, "out": out, "tensor_id_t": 5, "tensor_id_row": 3, "pre_quant": 0,
                                          "seed": 9, "col_sums": cs}], 1, 1, 0)
        for g, w, nm in zip(out, want, ("codes_t", "scales_t", "codes_row", "scales_row")):
            assert_same_bytes(g, w, nm)
        sums.append(host(cs))
    assert np.array_equal(sums[0], sums[1])
    ref = orc.column_sums(np.ascontiguousarray(x[:, :cols]))
    absref = np.abs(x[:, :cols]).astype(np.float64).sum(0)
    # every value passes at most 4 + 3 + 8 additions inside a 256-row block, then fewer than one per block plus 8
    tol = (32 + (rows + 255) // 256) * 2.0 ** -24 * absref
    assert np.all(np.abs(sums[0].astype(np.float64) - ref) <= tol + 1e-30), np.max(np.abs(sums[0] - ref) / (absref + 1e-300))
    # and bit for bit the FP32 sums in the order the interface documents (round to nearest in every
    # addition, although the stochastic quantizer around them runs under a directed rounding mode)
    assert np.array_equal(sums[0], orc.column_sums_f32_ordered(np.ascontiguousarray(x[:, :cols])))


def test_column_sums_in_a_batch_of_two(mx, orc):
    """Two tensors in one launch, only the second with column sums; X-type flags (row RTN, double quantization)."""
    xa = mixed_matrix(320, 256, seed=95, dtype="bf16")
    xb = mixed_matrix(544, 128, seed=96, dtype="bf16")
    outs, wants = [], []
    for x in (xa, xb):
        w = orc.quantize_transposed(x, round_t=1, tensor_id_t=6, pre_quant=1, round_row=0, tensor_id_row=1, seed=4)
        wants.append(w)
        outs.append(tuple(torch.empty(t.shape, dtype=torch.uint8, device="cuda") for t in w))
    cs = torch.zeros(128, device="cuda")
    mx.mx_quantize_transposed_batch(
        [{"src": dev(xa, "bf16"), "out": outs[0], "tensor_id_t": 6, "tensor_id_row": 1, "seed": 4},
         {"src": dev(xb, "bf16"), "out": outs[1], "tensor_id_t": 6, "tensor_id_row": 1, "seed": 4, "col_sums": cs}], 1, 0, 0)
    for out, want in zip(outs, wants):
        for g, w, nm in zip(out, want, ("codes_t", "scales_t", "codes_row", "scales_row")):
            assert_same_bytes(g, w, nm)
    ref = orc.column_sums(xb)
    assert np.all(np.abs(host(cs).astype(np.float64) - ref) <= 35 * 2.0 ** -24 * np.abs(xb).astype(np.float64).sum(0) + 1e-30)
    assert np.array_equal(host(cs), orc.column_sums_f32_ordered(xb))


# ------------------------------------------------- seed in device memory, graph replay ----

def test_device_seed_equals_host_seed(mx, orc):
    """A seed read from device memory by the kernel gives the bytes of the same seed passed by value."""
    x = mixed_matrix(288, 320, seed=71, dtype="bf16")
    X = dev(x, "bf16")
    for seed in (5, (0x7ABCDEF1 << 32) + 0x92345678, -3):
        want = orc.quantize_transposed(x, round_t=1, tensor_id_t=5, pre_quant=0, round_row=1, tensor_id_row=3,
                                       seed=seed & 0xFFFFFFFFFFFFFFFF)
        out = tuple(torch.empty(w.shape, dtype=torch.uint8, device="cuda") for w in want)
        seed_t = torch.tensor([seed], dtype=torch.int64, device="cuda")
        mx.mx_quantize_transposed_batch([{"src": X, "out": out, "tensor_id_t": 5, "tensor_id_row": 3, "pre_quant": 0,
                                          "seed": seed_t}], 1, 1, 0)
        for g, w, nm in zip(out, want, ("codes_t", "scales_t", "codes_row", "scales_row")):
            assert_same_bytes(g, w, "%s seed %d" % (nm, seed))


@pytest.mark.parametrize("qema", [False, True])
def test_layer_pass_recorded_into_a_graph(mx, orc, qema):
    """Forward + backward recorded once into a HIP graph with the seed in device memory, replayed with
    three seeds (eager work and synchronization between the replays): every replay's packed bytes and
    products equal the oracle's for the seed the word held at that replay."""
    import mx_workloads as wl
    N, D, C = 544, 256, 384
    X, W, dY = wl.linear_layer(N, D, C, seed=5, dtype="bf16", outliers=3)
    Xd, Wd, dYd = dev(X, "bf16"), dev(W, "bf16"), dev(dY, "bf16")
    step = mx.MxLinearStep(N, D, C, out_dtype=torch.float32, qema=qema, beta=0.0)
    seed_t = torch.zeros(1, dtype=torch.int64, device="cuda")
    step.forward(Xd, Wd, seed_t)                         # one eager pass first: code objects loaded and the
    step.backward(dYd, seed_t)                           # EMA state allocated before the recording starts
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step.forward(Xd, Wd, seed_t)
        step.backward(dYd, seed_t)
    for seed in (11, (9 << 32) + 4, 12):
        seed_t.fill_(seed)
        step.y.zero_(); step.dx.zero_(); step.dw.zero_(); step.dytq.zero_(); step.xtq.zero_(); step.wtq.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        xt, wt, dy = oracle_layer(orc, X, W, dY, seed=seed)
        _check_layer(mx, orc, step, xt, wt, dy, step.y, step.dx, step.dw, N, D, C, False, False,
                     "replay with seed %d" % seed)


def test_two_streams_give_the_single_stream_results(mx, orc):
    """Two layers run concurrently on two streams (separate buffers): every packed byte and every product
    value equals what the same calls give one after the other on one stream (the library holds no state)."""
    import mx_workloads as wl
    shapes = [(2048 + 32, 256, 384), (1024 + 96, 384, 256)]
    data = [wl.linear_layer(N, D, C, seed=40 + i, dtype="bf16", outliers=2) for i, (N, D, C) in enumerate(shapes)]
    dev_data = [tuple(dev(t, "bf16") for t in d) for d in data]

    def run(streams):
        steps = [mx.MxLinearStep(N, D, C, out_dtype=torch.float32) for (N, D, C) in shapes]
        torch.cuda.synchronize()
        for rep in range(3):                             # several rounds so that the two streams really overlap
            for st, (X, W, dY), s in zip(steps, dev_data, streams):
                with torch.cuda.stream(s):
                    st.forward(X, W, seed=21)
                    st.backward(dY, seed=21)
        torch.cuda.synchronize()
        return [[t.clone() for t in (st.xq, st.xtq, st.wtq, st.dyq, st.dytq, st.y, st.dx, st.dw)] for st in steps]

    main = torch.cuda.current_stream()
    serial = run([main, main])
    both = run([torch.cuda.Stream(), torch.cuda.Stream()])
    for a_layer, b_layer in zip(serial, both):
        for u, v in zip(a_layer, b_layer):
            assert torch.equal(u, v)
    xt, wt, dy = oracle_layer(orc, *data[0], seed=21)
    assert_same_bytes(both[0][1], xt[0], "Q6 under two streams")


@pytest.mark.parametrize("qema", [False, True])
def test_two_stream_schedule_of_a_layer_equals_forward_backward(mx, orc, qema):
    """MxLinearStep.step_two_streams (the schedule bench.py times: quant W, quant dY and dW on a second
    stream beside quant X, forward and dX) leaves every packed operand and every product exactly as
    forward() + backward() on one stream do, also when several layers follow one another without a
    synchronization in between; and they are the oracle's."""
    import mx_workloads as wl
    shapes = [(2048 + 32, 512, 768), (1024 + 96, 768, 256), (4096, 256, 512)]
    data = [wl.linear_layer(N, D, C, seed=60 + i, dtype="bf16", outliers=2) for i, (N, D, C) in enumerate(shapes)]
    dev_data = [tuple(dev(t, "bf16") for t in d) for d in data]
    names = ("xq", "xs", "xtq", "xts", "wq", "ws", "wtq", "wts", "dyq", "dys", "dytq", "dyts", "y", "dx", "dw")

    def run(two):
        steps = [mx.MxLinearStep(N, D, C, out_dtype=torch.bfloat16, qema=qema, beta=0.9) for (N, D, C) in shapes]
        side = torch.cuda.Stream()
        torch.cuda.synchronize()
        for rep in range(2):                                 # the second round also exercises the EMA update
            for st, (X, W, dY) in zip(steps, dev_data):
                if two:
                    st.step_two_streams(X, W, dY, 33 + rep, side)
                else:
                    st.forward(X, W, 33 + rep)
                    st.backward(dY, 33 + rep)
        torch.cuda.synchronize()
        return [[getattr(st, n).clone() for n in names] for st in steps]

    one, two = run(False), run(True)
    for a_layer, b_layer in zip(one, two):
        for n, u, v in zip(names, a_layer, b_layer):
            assert torch.equal(u, v), n
    if not qema:
        xt, wt, dy = oracle_layer(orc, *data[0], seed=34)
        got = dict(zip(names, two[0]))
        assert_same_bytes(got["xtq"], xt[0], "Q6 under the two-stream schedule")
        assert_same_bytes(got["dytq"], dy[0], "Q5 under the two-stream schedule")
        assert_same_bytes(got["wtq"], wt[0], "Q4 under the two-stream schedule")


# ------------------------------------------------- full size, bench launch configuration ----

@pytest.mark.parametrize("layer", ["qkv", "proj", "fc1", "fc2"])
def test_full_size_vit_base_layer(mx, orc, layer):
    """ViT-B/16 batch 256 (N = 50432), every layer of the block, bf16 sources, the exact calls, buffers
    and launch configuration bench.py times (one launch for X and W, bf16 Y and dX, FP32 dW through the
    K-split path): all packed bytes compared in full, products on 4096 sampled entries each."""
    import mx_workloads as wl
    li, N, D, C = _config_layer("vit_base_b256", layer)
    X, W, dY = wl.linear_layer(N, D, C, seed=li, dtype="bf16")
    step = mx.MxLinearStep(N, D, C, out_dtype=torch.bfloat16, dw_dtype=torch.float32)
    y = step.forward(dev(X, "bf16"), dev(W, "bf16"), seed=7 + li)
    dx, dw = step.backward(dev(dY, "bf16"), seed=7 + li)
    xt, wt, dy = oracle_layer(orc, X, W, dY, seed=7 + li)
    del X, W, dY
    _check_layer(mx, orc, step, xt, wt, dy, y, dx, dw, N, D, C, True, True, "vit_base " + layer)


# ------------------------------------------------- Q-Ramping: oscillation detection ----

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_oscillation_accumulate_and_ramping_factor(mx, orc, dtype):
    """dist_W / dist_Q (Sec. 6.1) over a weight walk with a window restart, then N_w of Algorithm 2:
    every state array bit-exact against the oracle at every step."""
    import mx_workloads as wl
    C, D = 544, 320                                    # rows not a multiple of the launch width, 10 groups per row
    state = mx.OscillationState(C, D)
    ost = {k: np.zeros((C, D), np.float32) for k in ("w_prev", "wq_prev", "dist_w", "dist_q")}
    for t, W in enumerate(wl.weight_walk(C, D, seed=9, steps=7, sigma=3e-3)):
        if dtype == "bf16":
            W = wl.round_to_bf16(W)
        if t == 3:
            W[5, :64] = 0.0                            # all-zero groups: w_Q = 0 with scale byte 98
        codes, scales = orc.quantize(W)
        restart = t in (0, 5)
        orc.oscillation_accumulate(W, codes, scales, ost, init=restart)
        gq = mx.mx_quantize(dev(W, dtype))
        assert_same_bytes(gq[0], codes, "codes step %d" % t)
        mx.mx_oscillation_accumulate(dev(W, dtype), gq[0], gq[1], state, init=restart)
        assert np.array_equal(host(state.dist_w), ost["dist_w"]), t
        assert np.array_equal(host(state.dist_q), ost["dist_q"]), t
        assert np.array_equal(host(state.w_prev), ost["w_prev"]), t
        assert_same_bytes(state.codes_prev, codes, "previous codes step %d" % t)
        assert_same_bytes(state.scales_prev, scales, "previous scales step %d" % t)
    assert ost["dist_q"].max() > 0
    for k1, k2, nmax in ((16.0, 5, 16), (0.37, 3, 100), (1.0, 1, 7)):
        want = orc.ramping_factor(ost["dist_w"], ost["dist_q"], k1, k2, nmax)
        got = host(mx.mx_ramping_factor(state.dist_w, state.dist_q, k1, k2, nmax))
        assert np.array_equal(got, want), (k1, k2, nmax)
    # degenerate trajectories: elements that never moved, and quantized jumps without master movement
    dw = np.array([[0.0, 0.0, 1e-30, 1.0]], np.float32)
    dq = np.array([[0.0, 0.5, 1.0, 0.0]], np.float32)
    want = orc.ramping_factor(dw, dq, 16.0, 5, 16)
    got = host(mx.mx_ramping_factor(dev(dw), dev(dq), 16.0, 5, 16))
    assert np.array_equal(got, want) and list(want[0]) == [1, 16, 16, 1]


# ------------------------------------------------- oscillation diagnostics (Sec. 4) ----

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("scale_mode", [0, 1])
def test_quant_confidence_bit_exact(mx, orc, dtype, scale_mode):
    """QuantConf of Sec. 4.2 per element and its histogram, bit-exact: weights of the layer's
    distribution, plus latent values planted on every threshold and cell centre, an all-zero group,
    tiny and huge groups, and a strided source."""
    import mx_workloads as wl
    C, D = 200, 352                                    # ragged against the 256-lane launch, 11 groups per row
    W = wl.weights(C, D, seed=31)
    planted = [0.25, -0.75, 1.25, -1.75, 2.5, -3.5, 5.0, 0.0, 0.5, -1.0, 1.5, 2.125, -3.0, 4.25, -6.0, 6.0, 5.999, 0.2499]
    W[0, :32] = 0.0
    W[0, 0] = 6.0 * 0.125
    W[0, 1:1 + len(planted)] = np.asarray(planted) * 0.125
    W[1, :32] = 0.0                                    # all-zero group
    W[2, 32:64] *= 1e-30                               # groups near the bottom and the top of FP32's range
    W[3, 32:64] *= 1e30
    W[4, 5] = 0.9                                      # an outlier that Eq. 2's scale truncates
    if dtype == "bf16":
        W = wl.round_to_bf16(W)
    want, want_hist = orc.quant_confidence(W, scale_mode, bins=50)
    hist = torch.zeros(50, dtype=torch.int64, device="cuda")
    got, _ = mx.mx_quant_confidence(dev(W, dtype), scale_mode, hist=hist)
    assert np.array_equal(host(got).view(np.uint32), want.view(np.uint32))
    assert np.array_equal(host(hist).astype(np.uint64), want_hist)
    if scale_mode == 0:
        assert np.all(want[0, 1:8] == 0.0) and np.all(want[0, 8:17] == 1.0)
    # histogram only, added to the counters already there; strided source
    big = np.zeros((C, D + 64), np.float32)
    big[:, :D] = W
    view = dev(big, dtype)[:, :D]
    _, h2 = mx.mx_quant_confidence(view, scale_mode, conf=False, hist=hist)
    assert np.array_equal(host(h2).astype(np.uint64), 2 * want_hist)
    got2, _ = mx.mx_quant_confidence(view, scale_mode)
    assert np.array_equal(host(got2), want)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_rate_of_change_matches_oracle(mx, orc, dtype):
    """Terms of r(X) (Sec. 4.1) over a weight walk: each term within 1e-12 relative of the oracle's
    FP64 value (only the order of the FP64 sums differs: n * 2^-53 bounds it far below that), the
    previous tensor bit-exact, the window sum and count kept on the device, reruns bit-identical."""
    import mx_workloads as wl
    C, D = 300, 328                                    # cols a multiple of 8 only
    state = mx.RateOfChangeState(C, D)
    xp = np.zeros((C, D), np.float32)
    terms = []
    for t, W in enumerate(wl.weight_walk(C, 352, seed=13, steps=6, sigma=2e-3)):
        W = np.ascontiguousarray(W[:, :D])
        if dtype == "bf16":
            W = wl.round_to_bf16(W)
        restart = t in (0, 4)
        if restart:
            xp[...] = W
            terms = []
        else:
            terms.append(orc.rate_of_change_term(W, xp))
        mx.mx_rate_of_change_step(dev(W, dtype), state, init=restart)
        res = host(state.result)
        assert np.array_equal(host(state.x_prev), xp), t
        assert res[2] == len(terms)
        if terms:
            assert abs(res[0] - terms[-1]) <= 1e-12 * terms[-1], (t, res[0], terms[-1])
            assert abs(res[1] - sum(terms)) <= 1e-12 * sum(terms)
            assert abs(state.rate() - sum(terms) / len(terms)) <= 1e-12
    assert terms and terms[-1] > 0
    # the same step from the same state gives the same bits
    a = mx.RateOfChangeState(C, D)
    b = mx.RateOfChangeState(C, D)
    W0, W1 = list(wl.weight_walk(C, 352, seed=14, steps=1, sigma=1e-2))[:2]
    for st in (a, b):
        mx.mx_rate_of_change_step(dev(np.ascontiguousarray(W0[:, :D])), st)
        mx.mx_rate_of_change_step(dev(np.ascontiguousarray(W1[:, :D])), st)
    assert host(a.result).tobytes() == host(b.result).tobytes()
    # an unchanged tensor: 0; a zero previous tensor: +infinity
    z = mx.RateOfChangeState(8, 32)
    mx.mx_rate_of_change_step(dev(np.zeros((8, 32), np.float32)), z)
    mx.mx_rate_of_change_step(dev(np.zeros((8, 32), np.float32)), z)
    assert host(z.result)[0] == 0.0
    mx.mx_rate_of_change_step(dev(np.ones((8, 32), np.float32)), z)
    assert host(z.result)[0] == np.inf


# ------------------------------------------------- Q-Ramping's customised AdamW (Algorithm 2) ----

@pytest.mark.parametrize("grad_dtype", ["f32", "bf16"])
def test_ramping_adamw_matches_oracle(mx, orc, grad_dtype):
    """T steps of the optimizer from the same start, GPU (FP32) against the oracle (FP64), each on its
    own state.  The integer state (steps held, updates made) must be identical; w, m, v agree within
    the FP32 rounding of the ~10 operations of an update, which adds per step at most about
    2^-23 |w| (the stored weight) + 2e-6 lr N_max (the update term) to |w_gpu - w_oracle|."""
    import mx_workloads as wl
    C, D, T = 96, 200, 14                               # 19200 elements: 18.75 workgroups of 1024
    lr, b1, b2, eps, wd = (float(np.float32(x)) for x in (2e-3, 0.9, 0.999, 1e-8, 0.05))
    rng = np.random.default_rng(77)
    W0 = wl.weights(C, 224, seed=41)[:, :D].copy()
    factor = np.ones((C, D), np.int32)
    osc = rng.random((C, D)) < 0.15                     # the paper's oscillating minority, here 15 %
    factor[osc] = rng.choice([2, 3, 6, 11, 16], int(osc.sum()))
    ost = orc.ramping_adamw_state(W0)
    w = dev(W0)
    st = mx.RampingAdamwState((C, D))
    fac = dev(factor)
    gmax = 0.0
    for t in range(T):
        g = (rng.standard_normal((C, D)) * 3e-3 * 10.0 ** rng.uniform(-1, 1)).astype(np.float32)
        if t == 5:
            g[:, :8] = 0.0
        if grad_dtype == "bf16":
            g = wl.round_to_bf16(g)
        if t == 9:                                      # a new detection: factors change under held gradients
            factor = np.where(rng.random((C, D)) < 0.5, factor, np.maximum(1, factor // 2)).astype(np.int32)
            fac = dev(factor)
        gmax = max(gmax, float(np.abs(g).max()))
        orc.ramping_adamw_step(ost, g, factor, lr, b1, b2, eps, wd)
        mx.mx_ramping_adamw_step(w, dev(g, grad_dtype), st, fac, lr, b1, b2, eps, wd)
        assert np.array_equal(host(st.acc_steps).ravel(), ost["acc_steps"]), t
        assert np.array_equal(host(st.updates).ravel(), ost["updates"]), t
        n = t + 1
        tol_w = n * (2.0 ** -23 * np.abs(W0).max() + 2e-6 * lr * 16)
        err_w = np.abs(host(w).ravel().astype(np.float64) - ost["w"]).max()
        assert err_w <= tol_w, (t, err_w, tol_w)
        err_m = np.abs(host(st.m).ravel().astype(np.float64) - ost["m"]).max()
        assert err_m <= n * 3e-7 * gmax, (t, err_m)
        err_v = np.abs(host(st.v).ravel().astype(np.float64) - ost["v"]).max()
        assert err_v <= n * 3e-7 * gmax ** 2, (t, err_v)
        err_a = np.abs(host(st.g_acc).ravel().astype(np.float64) - ost["g_acc"]).max()
        assert err_a <= 16 * 2.0 ** -23 * gmax, (t, err_a)
    assert ost["updates"].min() < ost["updates"].max()
    # plain AdamW (no factor): same bar, and the ramping state is not needed
    ost = orc.ramping_adamw_state(W0)
    w = dev(W0)
    st = mx.RampingAdamwState((C, D), ramping=False)
    for t in range(4):
        g = (rng.standard_normal((C, D)) * 3e-3).astype(np.float32)
        orc.ramping_adamw_step(ost, g, None, lr, b1, b2, eps, wd)
        mx.mx_ramping_adamw_step(w, dev(g), st, None, lr, b1, b2, eps, wd)
    assert np.all(host(st.updates) == 4)
    assert np.abs(host(w).ravel().astype(np.float64) - ost["w"]).max() <= 4 * (2.0 ** -23 * np.abs(W0).max() + 2e-6 * lr)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_transposed_batch_equals_separate_calls(mx, orc, dtype):
    """mx_quantize_transposed_batch on (activation, weight, a third ragged tensor): every output byte
    equals the separate calls' and the oracle's; the tensors differ in size class (wide tiles with a
    split last round, half tiles only), ids and seeds."""
    import mx_workloads as wl
    shapes = [(8192 + 96, 320), (96, 320), (160, 96)]
    srcs = [wl.activations(shapes[0][0], shapes[0][1], seed=3, outliers=3), wl.weights(shapes[1][0], shapes[1][1], seed=4),
            wl.weights(shapes[2][0], shapes[2][1], seed=5) * 50]
    if dtype == "bf16":
        srcs = [wl.round_to_bf16(a) for a in srcs]
    ids = [(6, 1, 11), (4, 2, 12), (9, 8, 13)]                      # (transposed id, row id, seed)
    devs = [dev(a, dtype) for a in srcs]
    jobs, outs = [], []
    for t, (r, c), (idt, idr, seed) in zip(devs, shapes, ids):
        out = tuple(torch.zeros(s, dtype=torch.uint8, device="cuda") for s in ((c, r // 2), (c, r // 32), (r, c // 2), (r, c // 32)))
        outs.append(out)
        jobs.append({"src": t, "out": out, "tensor_id_t": idt, "tensor_id_row": idr, "seed": seed})
    mx.mx_quantize_transposed_batch(jobs, mx.ROUND_SR, mx.ROUND_RTN)
    for a, t, out, (idt, idr, seed) in zip(srcs, devs, outs, ids):
        sep = mx.mx_quantize_transposed(t, mx.ROUND_SR, idt, 1, True, mx.ROUND_RTN, idr, seed=seed)
        want = orc.quantize_transposed(a, round_t=1, tensor_id_t=idt, pre_quant=1, round_row=0, tensor_id_row=idr, seed=seed)
        for got, s, w, nm in zip(out, sep, want, ("codes_t", "scales_t", "codes_row", "scales_row")):
            assert torch.equal(got, s), nm
            assert_same_bytes(got, w, "%s of tensor %s" % (nm, a.shape))


@pytest.mark.parametrize("rows,cols", [(16384, 1056), (16416, 1088)])
def test_transposed_wide_tiles_with_ragged_columns(mx, orc, rows, cols):
    """Tensors large enough for 256 x 128 macro tiles whose width is not a multiple of 128 (a last
    tile of 32 or 64 columns), with a last round issued as half tiles, and rows that are not a
    multiple of 256: every output byte against the oracle."""
    import mx_workloads as wl
    X = wl.round_to_bf16(wl.activations(rows, cols, seed=rows % 97, outliers=5))
    want = orc.quantize_transposed(X, round_t=1, tensor_id_t=6, pre_quant=1, round_row=0, tensor_id_row=1, seed=9)
    got = mx.mx_quantize_transposed(dev(X, "bf16"), mx.ROUND_SR, 6, 1, True, mx.ROUND_RTN, 1, seed=9)
    for g, w, nm in zip(got, want, ("codes_t", "scales_t", "codes_row", "scales_row")):
        assert_same_bytes(g, w, nm)
    want = orc.quantize_transposed(X, round_t=1, tensor_id_t=5, pre_quant=0, round_row=1, tensor_id_row=3, seed=9)
    got = mx.mx_quantize_transposed(dev(X, "bf16"), mx.ROUND_SR, 5, 0, True, mx.ROUND_SR, 3, seed=9)
    for g, w, nm in zip(got, want, ("codes_t", "scales_t", "codes_row", "scales_row")):
        assert_same_bytes(g, w, nm + " (both stochastic)")


# ------------------------------------------------- calibration helper ----

def test_calibration_mfma_counts_what_it_says(mx):
    """mx_calibration_mfma on the constant byte 0x22 (two codes of value 1): every MFMA adds 64 products
    of 1 x 1 to each accumulator entry, so after `it` iterations of two 64-K slices an entry holds
    128 it, and a lane's sink value (the sum of its 128 accumulator registers) is 128 * 128 * it,
    exactly (all integers below 2^24).  Pins the loop count behind the flop figure bench.py reports."""
    ops = torch.full((mx.CALIBRATION_MFMA_OPERAND_BYTES,), 0x22, dtype=torch.uint8, device="cuda")
    for it, wgs in ((1, 3), (7, 2)):
        sink = torch.zeros(wgs * 512, device="cuda")
        flops = mx.mx_calibration_mfma(ops, wgs, it, sink)
        torch.cuda.synchronize()
        assert flops == wgs * 8 * it * 16 * 2.0 * 32 * 32 * 64
        assert torch.all(sink == 128.0 * 128.0 * it)


# ------------------------------------------------- E3M0 elements (format ablation, Table 7) ----

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rnd", [0, 1])
@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("shape", [(256, 192), (37, 1056), (1, 32), (4100, 2080)])
def test_quantize_e3m0_rows(mx, orc, dtype, rnd, mode, shape):
    """The E3M0 quantizer against the oracle, bit for bit: both source types, both roundings, both scale
    rules; sizes from one group to more elements than one pass of the launch covers; midpoints of the
    E3M0 grid, all-zero groups and signed zeros planted; dequantized values too."""
    x = mixed_matrix(*shape, seed=30 + shape[0], dtype=dtype)
    if shape[1] >= 64:
        x[0, 32:40] = x[0, 40] * np.array([0.75, -0.75, 0.375, -0.375, 0.1875, -0.1875, 0.09375, 1.0], np.float32)
    want = orc.quantize_e3m0(x, round=rnd, scale_mode=mode, seed=78, tensor_id=5, index_base=8192)
    got = mx.mx_quantize_e3m0(dev(x, dtype), rnd, mode, seed=78, tensor_id=5, index_base=8192)
    assert_same_bytes(got[1], want[1], "scales")
    assert_same_bytes(got[0], want[0], "codes")
    deq = host(mx.mx_dequantize_e3m0(*got)).astype(np.float64)
    assert np.array_equal(deq, orc.dequantize_e3m0(*want))


def test_quantize_e3m0_extreme_values_and_strides(mx, orc):
    """Subnormals, the clamp at s = -127, the largest finite inputs, exact powers of two and their
    neighbours, quotients far below FP32's range; a strided view with a 64-bit seed and index base."""
    rows = 64
    x = np.zeros((rows, 64), np.float32)
    bits = np.array([0x00000001, 0x00000100, 0x007FFFFF, 0x00800000, 0x00800001, 0x00FFFFFF, 0x01000000,
                     0x3F800000, 0x3F800001, 0x3F7FFFFF, 0x7F7FFFFF, 0x7F000000, 0x7E800000, 0x41800000,
                     0x41800001, 0x417FFFFF], np.uint32)
    for i, b in enumerate(bits):
        x[i, 0] = np.array([b], np.uint32).view(np.float32)[0]
        x[i, 1:32] = x[i, 0] * np.linspace(-1, 1, 31, dtype=np.float32)
        x[i, 32] = -x[i, 0]
        x[i, 33:64] = x[i, 0] * np.float32(2.0) ** -np.arange(1, 32, dtype=np.float32) * 1.7
    rng = np.random.default_rng(1)
    x[16:48] = rng.standard_normal((32, 64)).astype(np.float32) * np.float32(2.0) ** rng.integers(-140, 120, (32, 1)).astype(np.float32)
    x[48:, ::32] = np.float32(2.0) ** rng.integers(0, 60, (16, 2)).astype(np.float32)
    tiny = np.float32(2.0) ** rng.integers(-149, -100, (16, 64)).astype(np.float32) * rng.choice(np.array([-1.0, 1.0], np.float32), (16, 64))
    mask = np.ones((16, 64), bool)
    mask[:, ::32] = False
    x[48:][mask] = tiny[mask]
    x = np.nan_to_num(x, posinf=3e38, neginf=-3e38)
    for rnd in (0, 1):
        for mode in (0, 1):
            for seed in (5, 6):
                want = orc.quantize_e3m0(x, round=rnd, scale_mode=mode, seed=seed, tensor_id=1)
                got = mx.mx_quantize_e3m0(dev(x), rnd, mode, seed=seed, tensor_id=1)
                assert_same_bytes(got[1], want[1], "scales r%d m%d" % (rnd, mode))
                assert_same_bytes(got[0], want[0], "codes r%d m%d" % (rnd, mode))
    big = mixed_matrix(64, 256, seed=4, dtype="bf16")
    seed = 0xDEADBEEF12345678
    want = orc.quantize_e3m0(big[:, 64:192], round=1, seed=seed, tensor_id=0xFFFFFFFF, index_base=(1 << 36) + 8)
    got = mx.mx_quantize_e3m0(dev(big, "bf16")[:, 64:192], 1, 0, seed=seed, tensor_id=0xFFFFFFFF, index_base=(1 << 36) + 8)
    assert_same_bytes(got[0], want[0], "strided codes")
    assert_same_bytes(got[1], want[1], "strided scales")


# ------------------------------------------------- fc1 with GELU and the next layer's quantizer fused ----

def _check_fused_quantizer(orc, P64, absref, P_gpu, got_c, got_s, scale_mode, tag):
    """The kernel quantizes A' = gelu_f32(P_gpu).  |A' - GELU(P64)| <= 1.13 |P_gpu - P64| + 2^-18 |A| + 2^-120
    (GELU's Lipschitz constant; FP32 erfc and its underflow), so: the product is within the product tolerance; every scale byte is one
    that a group maximum within that distance gives; and, under the kernel's scale, every dequantized value
    lies between round_D(A - tol) and round_D(A + tol) (round_D is monotone).  Where nothing is near a
    threshold this is bit equality with the oracle, and the check counts how often that is."""
    err = np.abs(P_gpu.astype(np.float64) - P64)
    assert np.all(err <= 1e-5 * absref), (tag, "product", np.max(err / (absref + 1e-300)))
    A = orc.gelu(P64)
    tol = 1.13 * err + 2.0 ** -18 * np.abs(A) + 2.0 ** -120          # the last term: FP32 erfc underflows near 1e-38
    want_c, want_s = orc.quantize(A.astype(np.float32), scale_mode=scale_mode)
    rows, cols = A.shape
    same_scale = got_s == want_s
    for r, gidx in zip(*np.nonzero(~same_scale)):
        seg = slice(32 * gidx, 32 * gidx + 32)
        lo = max(float(np.max(np.abs(A[r, seg]) - tol[r, seg])), 0.0)
        hi = float(np.max(np.abs(A[r, seg]) + tol[r, seg]))
        # a maximum of exactly 0 takes the epsilon rule (s = -29); any positive maximum up to hi takes its own
        s_ok = set(range(orc.shared_exponent(np.float32(lo), scale_mode) if lo > 0 else -127,
                         orc.shared_exponent(np.float32(hi), scale_mode) + 1))
        if lo == 0.0:
            s_ok.add(orc.shared_exponent(0.0, scale_mode))
        assert int(got_s[r, gidx]) - 127 in s_ok, (tag, "scale", r, gidx)
    got_v = orc.dequantize(got_c, got_s)
    exact = np.repeat(same_scale, 32, axis=1) & (got_v == orc.dequantize(want_c, want_s))
    S = np.repeat(2.0 ** (got_s.astype(np.float64) - 127), 32, axis=1)
    clamp = (lambda y: min(max(y, -6.0), 6.0)) if scale_mode == 1 else (lambda y: y)
    for r, c in zip(*np.nonzero(~exact)):
        lo = orc.e2m1_value(orc.round_rtn(np.float32(clamp((A[r, c] - tol[r, c]) / S[r, c])))) * S[r, c]
        hi = orc.e2m1_value(orc.round_rtn(np.float32(clamp((A[r, c] + tol[r, c]) / S[r, c])))) * S[r, c]
        assert lo <= got_v[r, c] <= hi, (tag, "code", r, c, A[r, c], tol[r, c], got_v[r, c], lo, hi)
    return float(exact.mean())


@pytest.mark.parametrize("scale_mode", [0, 1])
@pytest.mark.parametrize("N,C,D", [(320, 384, 512), (544, 416, 768), (256, 256, 1024)])
def test_linear_fwd_gelu_quant(mx, orc, N, C, D, scale_mode):
    """mx_linear_fwd_gelu_quant against the oracle's product -> GELU -> quantizer: edge rows and columns of
    the 256 x 256 tiles, a column count whose scale rows are not word-aligned, FP32 and bf16 pre-activation
    outputs; nearly all codes must equal the oracle's outright."""
    import mx_workloads as wl
    X, W, _ = wl.linear_layer(N, D, C, seed=50 + N, dtype="bf16", outliers=3)
    W = (W * 4).astype(np.float32)                           # pre-activations of order 1: both GELU branches
    rng = np.random.default_rng(N)
    bias = rng.standard_normal(C).astype(np.float32)
    bias[:32] = -30.0                                        # a whole group deep in GELU's negative tail
    xq, xs = orc.quantize(X)
    wq, ws = orc.quantize(W)
    P64, A64, _, _ = orc.linear_fwd_gelu_quant(xq, xs, wq, ws, bias, scale_mode)
    absref = np.abs(orc.dequantize(xq, xs)) @ np.abs(orc.dequantize(wq, ws)).T + np.abs(bias.astype(np.float64))[None, :]
    args = (dev(xq, "u8"), dev(xs, "u8"), dev(wq, "u8"), dev(ws, "u8"), dev(bias))
    y, aq, as_ = mx.mx_linear_fwd_gelu_quant(*args, out_dtype=torch.float32, scale_mode=scale_mode)
    frac = _check_fused_quantizer(orc, P64, absref, host(y), host(aq), host(as_), scale_mode, "fused %dx%dx%d" % (N, C, D))
    assert frac > 0.999, frac
    # the same codes with a bf16 pre-activation output (the quantizer sees the FP32 value either way), and the
    # pre-activation is what mx_linear_fwd_bias stores
    y16, aq16, as16 = mx.mx_linear_fwd_gelu_quant(*args, out_dtype=torch.bfloat16, scale_mode=scale_mode)
    assert torch.equal(aq16, aq) and torch.equal(as16, as_)
    assert torch.equal(y16, mx.mx_linear_fwd_bias(*args, out_dtype=torch.bfloat16))
    assert torch.equal(y, mx.mx_linear_fwd_bias(*args, out_dtype=torch.float32))
    # the next layer: its forward product takes (aq, as) as they are, its Q(6) re-quantizes them
    W2 = wl.weights(96, C, seed=3, dtype="bf16")
    w2q, w2s = orc.quantize(W2)
    y2 = mx.mx_linear_fwd(aq, as_, dev(w2q, "u8"), dev(w2s, "u8"), out_dtype=torch.float32)
    check_product(orc, y2, host(aq), host(as_), w2q, w2s, "next layer on fused codes")
    if N % 32 == 0:
        t = mx.mx_quantize_transposed(None, 1, 6, 1, False, row_in=(aq, as_), seed=4, shape=(N, C))
        Adq = orc.dequantize(host(aq), host(as_)).astype(np.float32)
        want_t = orc.quantize_transposed(Adq, round_t=1, tensor_id_t=6, pre_quant=0, want_row=False, seed=4)
        assert_same_bytes(t[0], want_t[0], "Q6 of the fused codes")
        assert_same_bytes(t[1], want_t[1], "S6 of the fused codes")


def test_linear_fwd_gelu_quant_full_size_fc1(mx, orc):
    """ViT-B/16 batch 256 fc1 (50432 x 768 -> 3072) through the fused entry point: 384 sampled rows (first,
    last, random) checked in full against the oracle."""
    import mx_workloads as wl
    N, D, C = 50432, 768, 3072
    X, W, _ = wl.linear_layer(N, D, C, seed=2, dtype="bf16")
    W = (W * 2).astype(np.float32)
    bias = np.random.default_rng(5).standard_normal(C).astype(np.float32) * 0.5
    xq, xs = orc.quantize(X)
    wq, ws = orc.quantize(W)
    del X
    y, aq, as_ = mx.mx_linear_fwd_gelu_quant(dev(xq, "u8"), dev(xs, "u8"), dev(wq, "u8"), dev(ws, "u8"), dev(bias),
                                             out_dtype=torch.float32)
    rows = np.unique(np.concatenate([[0, 1, 255, 256, N - 257, N - 256, N - 1], np.random.default_rng(6).integers(0, N, 380)]))
    P64, A64, _, _ = orc.linear_fwd_gelu_quant(xq[rows], xs[rows], wq, ws, bias)
    absref = np.abs(orc.dequantize(xq[rows], xs[rows])) @ np.abs(orc.dequantize(wq, ws)).T + np.abs(bias.astype(np.float64))[None, :]
    idx = torch.from_numpy(rows).cuda()
    frac = _check_fused_quantizer(orc, P64, absref, host(y[idx]), host(aq[idx]), host(as_[idx]), 0, "fused fc1")
    assert frac > 0.999, frac
