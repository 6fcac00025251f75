"""ctypes loader for the CPU oracle (mx_oracle.c).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
module; only tests, the smoke check and the benchmark's cpu_baseline leg do.
All arrays are numpy; FP32 in, uint8 codes/scales and FP64 products out.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mx_oracle.c")
_LIB = os.path.join(_HERE, "libmx_oracle.so")

ROUND_RTN, ROUND_SR = 0, 1
SCALE_TRUNCFREE, SCALE_FLOOR = 0, 1


def build(force=False):
    """Compile mx_oracle.c with gcc into libmx_oracle.so next to it."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)
            and os.path.getmtime(_LIB) >= os.path.getmtime(os.path.join(_HERE, "mx_oracle.h"))):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
           "-Wall", "-Wextra", _SRC, "-o", _LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None

_u8p = ctypes.POINTER(ctypes.c_uint8)
_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_i32p = ctypes.POINTER(ctypes.c_int32)
_i64p = ctypes.POINTER(ctypes.c_int64)
_u32p = ctypes.POINTER(ctypes.c_uint32)
_i64, _u64, _u32, _int = ctypes.c_int64, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        L.orc_e2m1_value.restype = ctypes.c_double
        L.orc_e2m1_value.argtypes = [_int]
        L.orc_philox4x32_10.restype = None
        L.orc_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
        L.orc_sr_bits.restype = _u32
        L.orc_sr_bits.argtypes = [_u64, _u32, _u64]
        L.orc_shared_exponent.restype = _int
        L.orc_shared_exponent.argtypes = [ctypes.c_float, _int]
        L.orc_round_rtn.restype = _int
        L.orc_round_rtn.argtypes = [ctypes.c_float]
        L.orc_round_sr.restype = _int
        L.orc_round_sr.argtypes = [ctypes.c_float, _u32]
        L.orc_round_ema.restype = _int
        L.orc_round_ema.argtypes = [ctypes.c_float, ctypes.c_float]
        L.orc_gelu.restype = None
        L.orc_gelu.argtypes = [_f64p, _i64, _f64p]
        L.orc_e3m0_value.restype = ctypes.c_double
        L.orc_e3m0_value.argtypes = [_int]
        L.orc_shared_exponent_e3m0.restype = _int
        L.orc_shared_exponent_e3m0.argtypes = [ctypes.c_float, _int]
        L.orc_round_rtn_e3m0.restype = _int
        L.orc_round_rtn_e3m0.argtypes = [ctypes.c_float]
        L.orc_round_sr_e3m0.restype = _int
        L.orc_round_sr_e3m0.argtypes = [ctypes.c_float, _u32]
        L.orc_quantize_e3m0.restype = None
        L.orc_quantize_e3m0.argtypes = [_f32p, _i64, _i64, _i64, _u8p, _u8p, _int, _int, _u64, _u32, _u64]
        L.orc_dequantize_e3m0.restype = None
        L.orc_dequantize_e3m0.argtypes = [_u8p, _u8p, _i64, _i64, _f64p]
        L.orc_quantize.restype = None
        L.orc_quantize.argtypes = [_f32p, _i64, _i64, _i64, _u8p, _u8p, _int, _int, _u64, _u32, _u64]
        L.orc_quantize_transposed.restype = None
        L.orc_quantize_transposed.argtypes = [_f32p, _i64, _i64, _i64, _u8p, _u8p, _int, _u32, _int,
                                              _u8p, _u8p, _int, _u32, _u8p, _u8p, _int, _u64, _u64]
        L.orc_ema_weight_quant.restype = None
        L.orc_ema_weight_quant.argtypes = [_f32p, _f32p, ctypes.c_float, _int, _i64, _i64, _i64,
                                           _u8p, _u8p, _int]
        L.orc_dequantize.restype = None
        L.orc_dequantize.argtypes = [_u8p, _u8p, _i64, _i64, _f64p]
        L.orc_gemm_f64.restype = None
        L.orc_gemm_f64.argtypes = [_u8p, _u8p, _u8p, _u8p, _i64, _i64, _i64, _f64p]
        L.orc_gemm_f64_sampled.restype = None
        L.orc_gemm_f64_sampled.argtypes = [_u8p, _u8p, _u8p, _u8p, _i64, _i64, _i64,
                                           _i64p, _i64p, _i64, _f64p, _f64p]
        L.orc_num_threads.restype = _int
        L.orc_num_threads.argtypes = []
        L.orc_oscillation_accumulate.restype = None
        L.orc_oscillation_accumulate.argtypes = [_f32p, _i64, _i64, _i64, _u8p, _u8p, _f32p, _f32p, _f32p, _f32p, _int]
        L.orc_quant_confidence.restype = None
        L.orc_quant_confidence.argtypes = [_f32p, _i64, _i64, _i64, _int, _f32p, ctypes.POINTER(ctypes.c_uint64), _int]
        L.orc_column_sums.restype = None
        L.orc_column_sums.argtypes = [_f32p, _i64, _i64, _i64, _f64p]
        L.orc_rate_of_change_term.restype = ctypes.c_double
        L.orc_rate_of_change_term.argtypes = [_f32p, _i64, _i64, _i64, _f32p]
        L.orc_ramping_adamw_step.restype = None
        L.orc_ramping_adamw_step.argtypes = [_f64p, _f64p, _i64, _f64p, _f64p, _f64p, _i32p, _i32p, _i32p,
                                             ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_double,
                                             ctypes.c_double]
        L.orc_ramping_factor.restype = None
        L.orc_ramping_factor.argtypes = [_f32p, _f32p, _i64, ctypes.c_float, _int, _int, ctypes.POINTER(ctypes.c_int32)]
        _lib = L
    return _lib


def _p(a, typ):
    return a.ctypes.data_as(typ) if a is not None else typ()


def _f32(a):
    a = np.asarray(a)
    assert a.dtype == np.float32 and a.ndim == 2 and a.strides[1] == 4
    return a


def _u8(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint8
    return a


def e2m1_value(code):
    return lib().orc_e2m1_value(int(code))


def philox4x32_10(ctr, key):
    c = (ctypes.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
    k = (ctypes.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    o = (ctypes.c_uint32 * 4)()
    lib().orc_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def sr_bits(seed, tensor_id, e):
    return int(lib().orc_sr_bits(int(seed), int(tensor_id), int(e)))


def shared_exponent(M, scale_mode=SCALE_TRUNCFREE):
    return int(lib().orc_shared_exponent(float(M), int(scale_mode)))


def round_rtn(y):
    return int(lib().orc_round_rtn(float(y)))


def round_sr(y, r16):
    return int(lib().orc_round_sr(float(y), int(r16)))


def round_ema(y, z):
    return int(lib().orc_round_ema(float(y), float(z)))


def quantize(src, round=ROUND_RTN, scale_mode=SCALE_TRUNCFREE, seed=0, tensor_id=0, index_base=0):
    """1x32 groups along the columns -> (codes[rows, cols/2], scales[rows, cols/32])."""
    src = _f32(src)
    rows, cols = src.shape
    assert cols % 32 == 0
    ld = src.strides[0] // 4
    codes = np.zeros((rows, cols // 2), np.uint8)
    scales = np.zeros((rows, cols // 32), np.uint8)
    lib().orc_quantize(_p(src, _f32p), rows, cols, ld, _p(codes, _u8p), _p(scales, _u8p),
                       int(round), int(scale_mode), int(seed), int(tensor_id), int(index_base))
    return codes, scales


def quantize_transposed(src, round_t=ROUND_SR, tensor_id_t=0, pre_quant=1, want_row=True,
                        round_row=ROUND_RTN, tensor_id_row=0, row_in=None,
                        scale_mode=SCALE_TRUNCFREE, seed=0, index_base=0):
    """32x1 groups down the rows, stored transposed.

    Returns (codes_t[cols, rows/2], scales_t[cols, rows/32], codes_row, scales_row);
    the last two are None unless want_row.
    """
    src = _f32(src)
    rows, cols = src.shape
    assert rows % 32 == 0
    ld = src.strides[0] // 4
    codes_t = np.zeros((cols, rows // 2), np.uint8)
    scales_t = np.zeros((cols, rows // 32), np.uint8)
    codes_row = scales_row = None
    if want_row:
        codes_row = np.zeros((rows, cols // 2), np.uint8)
        scales_row = np.zeros((rows, cols // 32), np.uint8)
    rc_in = rs_in = None
    if row_in is not None:
        rc_in, rs_in = _u8(row_in[0]), _u8(row_in[1])
    lib().orc_quantize_transposed(_p(src, _f32p), rows, cols, ld, _p(codes_t, _u8p), _p(scales_t, _u8p),
                                  int(round_t), int(tensor_id_t), int(pre_quant),
                                  _p(codes_row, _u8p), _p(scales_row, _u8p),
                                  int(round_row), int(tensor_id_row),
                                  _p(rc_in, _u8p), _p(rs_in, _u8p),
                                  int(scale_mode), int(seed), int(index_base))
    return codes_t, scales_t, codes_row, scales_row


def ema_weight_quant(w, w_ema, beta=0.998, update_ema=1, scale_mode=SCALE_TRUNCFREE):
    """Q-EMA.  w_ema (float32, same shape as w) is updated in place."""
    w = _f32(w)
    assert w_ema.dtype == np.float32 and w_ema.shape == w.shape and w_ema.strides == w.strides
    rows, cols = w.shape
    ld = w.strides[0] // 4
    codes = np.zeros((rows, cols // 2), np.uint8)
    scales = np.zeros((rows, cols // 32), np.uint8)
    lib().orc_ema_weight_quant(_p(w, _f32p), _p(w_ema, _f32p), float(beta), int(update_ema),
                               rows, cols, ld, _p(codes, _u8p), _p(scales, _u8p), int(scale_mode))
    return codes, scales


def dequantize(codes, scales):
    codes, scales = _u8(codes), _u8(scales)
    rows, cols = codes.shape[0], codes.shape[1] * 2
    out = np.zeros((rows, cols), np.float64)
    lib().orc_dequantize(_p(codes, _u8p), _p(scales, _u8p), rows, cols, _p(out, _f64p))
    return out


def gelu(x):
    """GELU(x) = x * Phi(x), FP64, element-wise."""
    x = np.ascontiguousarray(x, np.float64)
    out = np.empty_like(x)
    lib().orc_gelu(_p(x.reshape(-1), _f64p), x.size, _p(out.reshape(-1), _f64p))
    return out


def linear_fwd_gelu_quant(xq, xs, wq, ws, bias, scale_mode=SCALE_TRUNCFREE):
    """The first MLP layer followed by GELU and the next layer's forward quantizer, step by step:
    P = Q1(X) . Q2(W)^T + bias (FP64), A = GELU(P) (FP64), then the 1x32 round_D quantizer on A rounded
    to FP32.  Returns (P, A, codes, scales)."""
    P = gemm_f64(xq, xs, wq, ws) + np.asarray(bias, np.float64)[None, :]
    A = gelu(P)
    codes, scales = quantize(A.astype(np.float32), round=ROUND_RTN, scale_mode=scale_mode)
    return P, A, codes, scales


# ---- E3M0 elements (Table 7's format ablation) ----

def e3m0_value(code):
    return lib().orc_e3m0_value(int(code))


def shared_exponent_e3m0(M, scale_mode=SCALE_TRUNCFREE):
    return int(lib().orc_shared_exponent_e3m0(float(M), int(scale_mode)))


def round_rtn_e3m0(y):
    return int(lib().orc_round_rtn_e3m0(float(y)))


def round_sr_e3m0(y, r16):
    return int(lib().orc_round_sr_e3m0(float(y), int(r16)))


def quantize_e3m0(src, round=ROUND_RTN, scale_mode=SCALE_TRUNCFREE, seed=0, tensor_id=0, index_base=0):
    """1x32 groups along the columns, E3M0 elements -> (codes[rows, cols/2], scales[rows, cols/32])."""
    src = _f32(src)
    rows, cols = src.shape
    assert cols % 32 == 0
    ld = src.strides[0] // 4
    codes = np.zeros((rows, cols // 2), np.uint8)
    scales = np.zeros((rows, cols // 32), np.uint8)
    lib().orc_quantize_e3m0(_p(src, _f32p), rows, cols, ld, _p(codes, _u8p), _p(scales, _u8p),
                            int(round), int(scale_mode), int(seed), int(tensor_id), int(index_base))
    return codes, scales


def dequantize_e3m0(codes, scales):
    codes, scales = _u8(codes), _u8(scales)
    rows, cols = codes.shape[0], codes.shape[1] * 2
    out = np.zeros((rows, cols), np.float64)
    lib().orc_dequantize_e3m0(_p(codes, _u8p), _p(scales, _u8p), rows, cols, _p(out, _f64p))
    return out


def gemm_f64(a_codes, a_scales, b_codes, b_scales):
    """C[m, n] = A[m, k] . B[n, k]^T on dequantized operands, FP64."""
    a_codes, a_scales, b_codes, b_scales = map(_u8, (a_codes, a_scales, b_codes, b_scales))
    m, k = a_codes.shape[0], a_codes.shape[1] * 2
    n = b_codes.shape[0]
    assert b_codes.shape[1] * 2 == k
    c = np.zeros((m, n), np.float64)
    lib().orc_gemm_f64(_p(a_codes, _u8p), _p(a_scales, _u8p), _p(b_codes, _u8p), _p(b_scales, _u8p),
                       m, n, k, _p(c, _f64p))
    return c


def gemm_f64_sampled(a_codes, a_scales, b_codes, b_scales, ii, jj):
    """Entries (ii[t], jj[t]) of the same product, plus sum_k |a||b| for each."""
    a_codes, a_scales, b_codes, b_scales = map(_u8, (a_codes, a_scales, b_codes, b_scales))
    m, k = a_codes.shape[0], a_codes.shape[1] * 2
    n = b_codes.shape[0]
    ii = np.ascontiguousarray(ii, np.int64)
    jj = np.ascontiguousarray(jj, np.int64)
    out = np.zeros(ii.shape[0], np.float64)
    aout = np.zeros(ii.shape[0], np.float64)
    lib().orc_gemm_f64_sampled(_p(a_codes, _u8p), _p(a_scales, _u8p), _p(b_codes, _u8p), _p(b_scales, _u8p),
                               m, n, k, _p(ii, _i64p), _p(jj, _i64p), ii.shape[0],
                               _p(out, _f64p), _p(aout, _f64p))
    return out, aout


def num_threads():
    return int(lib().orc_num_threads())


def oscillation_accumulate(w, codes, scales, state, init=False):
    """One step of Q-Ramping's oscillation detection.  state = dict of float32 arrays
    w_prev, wq_prev, dist_w, dist_q (shape of w), updated in place."""
    w = _f32(w)
    codes, scales = _u8(codes), _u8(scales)
    rows, cols = w.shape
    for k in ("w_prev", "wq_prev", "dist_w", "dist_q"):
        a = state[k]
        assert a.dtype == np.float32 and a.shape == (rows, cols) and a.flags["C_CONTIGUOUS"]
    lib().orc_oscillation_accumulate(_p(w, _f32p), rows, cols, w.strides[0] // 4, _p(codes, _u8p), _p(scales, _u8p),
                                     _p(state["w_prev"], _f32p), _p(state["wq_prev"], _f32p),
                                     _p(state["dist_w"], _f32p), _p(state["dist_q"], _f32p), int(bool(init)))
    return state


def ramping_factor(dist_w, dist_q, k1=16.0, k2=5, n_max=16):
    """N_w of Algorithm 2 (Q-Ramping) per element, int32."""
    dw = np.ascontiguousarray(dist_w, np.float32).ravel()
    dq = np.ascontiguousarray(dist_q, np.float32).ravel()
    out = np.zeros(dw.shape, np.int32)
    lib().orc_ramping_factor(_p(dw, _f32p), _p(dq, _f32p), dw.size, float(k1), int(k2), int(n_max),
                             out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    return out.reshape(np.shape(dist_w))



def quant_confidence(w, scale_mode=SCALE_TRUNCFREE, bins=0):
    """QuantConf of Sec. 4.2 per element (float32, shape of w); with bins > 0 also the histogram
    (uint64[bins]) of the confidences."""
    w = _f32(w)
    rows, cols = w.shape
    conf = np.zeros((rows, cols), np.float32)
    hist = np.zeros(bins, np.uint64) if bins > 0 else None
    lib().orc_quant_confidence(_p(w, _f32p), rows, cols, w.strides[0] // 4, int(scale_mode), _p(conf, _f32p),
                               hist.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)) if bins > 0 else None, int(bins))
    return (conf, hist) if bins > 0 else conf


def column_sums(x):
    """out[c] = sum over r of x[r][c], FP64 (the bias gradient when x is dY)."""
    x = _f32(x)
    rows, cols = x.shape
    out = np.zeros(cols, np.float64)
    lib().orc_column_sums(_p(x, _f32p), rows, cols, x.strides[0] // 4, _p(out, _f64p))
    return out


def column_sums_f32_ordered(x):
    """The same column sums in FP32, added in the one order the library's interface documents for its
    col_sums output (so that the kernel's result can be compared bit for bit, rounding mode included):
    rows in blocks of 256, a block in tiles of 32 rows; inside a tile four consecutive rows are added
    left to right, g_i = ((x[4i] + x[4i+1]) + x[4i+2]) + x[4i+3], the eight g_i pairwise as a balanced
    tree ((g0 + g1) + (g2 + g3)) + ((g4 + g5) + (g6 + g7)); the tiles of a block in index order; the
    blocks as eight contiguous runs of ceil(blocks / 8), each run added in index order starting from 0,
    and the eight runs in index order.  Every addition rounds to nearest even.  rows % 32 == 0."""
    x = _f32(x)
    rows, cols = x.shape
    assert rows % 32 == 0
    f = np.float32
    blocks = (rows + 255) // 256
    partial = np.zeros((blocks, cols), f)
    for b in range(blocks):
        r0, r1 = b * 256, min(rows, b * 256 + 256)
        acc = None
        for t0 in range(r0, r1, 32):
            g = [((x[t0 + 4 * i] + x[t0 + 4 * i + 1]) + x[t0 + 4 * i + 2]) + x[t0 + 4 * i + 3] for i in range(8)]
            tile = ((g[0] + g[1]) + (g[2] + g[3])) + ((g[4] + g[5]) + (g[6] + g[7]))
            acc = tile if acc is None else (acc + tile).astype(f)
        partial[b] = acc
    per = (blocks + 7) // 8
    runs = []
    for p in range(8):
        s = np.zeros(cols, f)
        for b in range(min(blocks, p * per), min(blocks, p * per + per)):
            s = (s + partial[b]).astype(f)
        runs.append(s)
    out = runs[0]
    for p in range(1, 8):
        out = (out + runs[p]).astype(f)
    return out


def rate_of_change_term(x, x_prev):
    """||x - x_prev||_F / ||x_prev||_F (Sec. 4.1), FP64; x_prev (float32, dense, shape of x) is then set to x."""
    x = _f32(x)
    rows, cols = x.shape
    assert x_prev.dtype == np.float32 and x_prev.shape == (rows, cols) and x_prev.flags["C_CONTIGUOUS"]
    return float(lib().orc_rate_of_change_term(_p(x, _f32p), rows, cols, x.strides[0] // 4, _p(x_prev, _f32p)))


def ramping_adamw_state(w):
    """Fresh optimizer state for weights w: dict of float64 w, m, v, g_acc and int32 acc_steps, updates."""
    w = np.array(w, np.float64).ravel()
    z = lambda t: np.zeros(w.shape, t)
    return {"w": w, "m": z(np.float64), "v": z(np.float64), "g_acc": z(np.float64),
            "acc_steps": z(np.int32), "updates": z(np.int32)}


def ramping_adamw_step(state, grad, factor=None, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01):
    """One step of Q-Ramping's customised AdamW (Algorithm 2) on the state, in place."""
    g = np.ascontiguousarray(np.asarray(grad, np.float64).ravel())
    n = state["w"].size
    assert g.size == n
    f = None
    if factor is not None:
        f = np.ascontiguousarray(np.asarray(factor, np.int32).ravel())
        assert f.size == n
    lib().orc_ramping_adamw_step(_p(state["w"], _f64p), _p(g, _f64p), n, _p(state["m"], _f64p), _p(state["v"], _f64p),
                                 _p(state["g_acc"], _f64p), _p(f, _i32p), _p(state["acc_steps"], _i32p),
                                 _p(state["updates"], _i32p), float(lr), float(beta1), float(beta2), float(eps),
                                 float(weight_decay))
    return state
