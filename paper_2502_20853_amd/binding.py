"""Thin Python binding of the C ABI in include/mxfp4.h.

Argument marshalling only: torch supplies device memory and the current HIP
stream; every step of the path runs in the library's kernels.  The functions
have the same names as the C entry points.  A missing or unloadable library is
an error -- there is no fallback path.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmxfp4_hip.so")

MX_OK = 0
MX_ERR_NULL, MX_ERR_SHAPE, MX_ERR_DTYPE, MX_ERR_MODE = -1, -2, -3, -4
MX_ERR_ALIGN, MX_ERR_WORKSPACE, MX_ERR_HIP = -5, -6, -7
_ERR_NAMES = {-1: "MX_ERR_NULL", -2: "MX_ERR_SHAPE", -3: "MX_ERR_DTYPE", -4: "MX_ERR_MODE",
              -5: "MX_ERR_ALIGN", -6: "MX_ERR_WORKSPACE", -7: "MX_ERR_HIP"}

DTYPE_F32, DTYPE_BF16 = 0, 1
ROUND_RTN, ROUND_SR = 0, 1
SCALE_TRUNCFREE, SCALE_FLOOR = 0, 1
GEMM_FWD, GEMM_BWD_DX, GEMM_BWD_DW = 0, 1, 2

EXPORTS = ["mx_quantize", "mx_quantize_e3m0", "mx_dequantize_e3m0", "mx_quantize_transposed", "mx_quantize_transposed_batch", "mx_column_sum_workspace_bytes", "mx_linear_fwd", "mx_linear_fwd_bias", "mx_linear_fwd_gelu_quant", "mx_linear_bwd_dx",
           "mx_linear_bwd_dw", "mx_linear_bwd_dw_noalloc", "mx_ema_weight_quant", "mx_linear_workspace_bytes",
           "mx_oscillation_accumulate", "mx_ramping_factor",
           "mx_ramping_adamw_step", "mx_quant_confidence", "mx_rate_of_change_workspace_bytes", "mx_rate_of_change_step",
           "mx_dequantize", "mx_calibration_copy", "mx_calibration_mfma", "mx_last_hip_error", "mx_version"]


class _TransposedJob(ctypes.Structure):
    """mx_transposed_job of include/mxfp4.h."""
    _fields_ = [("src", ctypes.c_void_p), ("dtype", ctypes.c_int), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("ld", ctypes.c_int64), ("codes_t", ctypes.c_void_p), ("scales_t", ctypes.c_void_p),
                ("tensor_id_t", ctypes.c_uint32), ("pre_quant", ctypes.c_int), ("codes_row", ctypes.c_void_p),
                ("scales_row", ctypes.c_void_p), ("tensor_id_row", ctypes.c_uint32),
                ("row_codes_in", ctypes.c_void_p), ("row_scales_in", ctypes.c_void_p),
                ("seed", ctypes.c_uint64), ("index_base", ctypes.c_uint64), ("seed_dev", ctypes.c_void_p),
                ("col_sums", ctypes.c_void_p), ("col_sum_workspace", ctypes.c_void_p)]


class MxError(RuntimeError):
    def __init__(self, fn, code, hip=0):
        self.code = code
        msg = "%s failed: %s (%d)" % (fn, _ERR_NAMES.get(code, "?"), code)
        if code == MX_ERR_HIP:
            msg += ", hipError_t %d" % hip
        super().__init__(msg)


_lib = None


def lib():
    """Load the HIP library (built by paper_2502_20853_amd.build); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("HIP library %s is not built: run `python -m paper_2502_20853_amd.build` "
                           "(or __graft_entry__.build())" % LIB_PATH)
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, u64, u32, ci, sz, f32 = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64, ctypes.c_uint32,
                                      ctypes.c_int, ctypes.c_size_t, ctypes.c_float)
    L.mx_quantize.restype = ci
    L.mx_quantize.argtypes = [vp, ci, i64, i64, i64, vp, vp, ci, ci, u64, u32, u64, vp]
    L.mx_quantize_e3m0.restype = ci
    L.mx_quantize_e3m0.argtypes = [vp, ci, i64, i64, i64, vp, vp, ci, ci, u64, u32, u64, vp]
    L.mx_dequantize_e3m0.restype = ci
    L.mx_dequantize_e3m0.argtypes = [vp, vp, i64, i64, vp, vp]
    L.mx_quantize_transposed.restype = ci
    L.mx_quantize_transposed.argtypes = [vp, ci, i64, i64, i64, vp, vp, ci, u32, ci, vp, vp, ci, u32,
                                         vp, vp, ci, u64, u64, vp]
    for name in ("mx_linear_fwd", "mx_linear_bwd_dx", "mx_linear_bwd_dw"):
        fn = getattr(L, name)
        fn.restype = ci
        fn.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, ci, i64, vp, sz, vp]
    L.mx_linear_bwd_dw_noalloc.restype = ci
    L.mx_linear_bwd_dw_noalloc.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, ci, i64, vp]
    L.mx_column_sum_workspace_bytes.restype = sz
    L.mx_column_sum_workspace_bytes.argtypes = [i64, i64]
    L.mx_linear_fwd_bias.restype = ci
    L.mx_linear_fwd_bias.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, vp, ci, i64, vp, sz, vp]
    L.mx_linear_fwd_gelu_quant.restype = ci
    L.mx_linear_fwd_gelu_quant.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, vp, ci, i64, vp, vp, ci, vp]
    L.mx_ema_weight_quant.restype = ci
    L.mx_ema_weight_quant.argtypes = [vp, ci, vp, f32, ci, i64, i64, i64, vp, vp, ci, vp]
    L.mx_linear_workspace_bytes.restype = sz
    L.mx_linear_workspace_bytes.argtypes = [ci, i64, i64, i64]
    L.mx_oscillation_accumulate.restype = ci
    L.mx_oscillation_accumulate.argtypes = [vp, ci, i64, i64, i64, vp, vp, vp, vp, vp, vp, vp, ci, vp]
    L.mx_ramping_factor.restype = ci
    L.mx_ramping_factor.argtypes = [vp, vp, i64, f32, ci, ci, vp, vp]
    L.mx_ramping_adamw_step.restype = ci
    L.mx_ramping_adamw_step.argtypes = [vp, vp, ci, i64, vp, vp, vp, vp, vp, vp, f32, f32, f32, f32, f32, vp]
    L.mx_quant_confidence.restype = ci
    L.mx_quant_confidence.argtypes = [vp, ci, i64, i64, i64, ci, vp, vp, ci, vp]
    L.mx_rate_of_change_workspace_bytes.restype = sz
    L.mx_rate_of_change_workspace_bytes.argtypes = []
    L.mx_rate_of_change_step.restype = ci
    L.mx_rate_of_change_step.argtypes = [vp, ci, i64, i64, i64, vp, ci, vp, sz, vp, vp]
    L.mx_dequantize.restype = ci
    L.mx_dequantize.argtypes = [vp, vp, i64, i64, vp, vp]
    L.mx_calibration_copy.restype = ci
    L.mx_calibration_copy.argtypes = [vp, vp, sz, vp]
    L.mx_calibration_mfma.restype = ci
    L.mx_calibration_mfma.argtypes = [vp, ci, ci, vp, vp]
    L.mx_last_hip_error.restype = ci
    L.mx_last_hip_error.argtypes = []
    L.mx_version.restype = ctypes.c_char_p
    L.mx_version.argtypes = []
    _lib = L
    return L


def _check(fn, rc):
    if rc != MX_OK:
        raise MxError(fn, rc, lib().mx_last_hip_error() if rc == MX_ERR_HIP else 0)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _src_dtype(t):
    if t.dtype == torch.float32:
        return DTYPE_F32
    if t.dtype == torch.bfloat16:
        return DTYPE_BF16
    raise TypeError("source must be float32 or bfloat16, got %s" % t.dtype)


def _matrix(t):
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError("expected a 2-D tensor with unit column stride")
    return t.shape[0], t.shape[1], t.stride(0)


def _u8(shape, device):
    return torch.empty(shape, dtype=torch.uint8, device=device)


def mx_version():
    return lib().mx_version().decode()


def mx_quantize(src, round=ROUND_RTN, scale_mode=SCALE_TRUNCFREE, seed=0, tensor_id=0, index_base=0,
                out=None, stream=None):
    """1x32 groups along the columns.  Returns (codes[rows, cols/2], scales[rows, cols/32])."""
    rows, cols, ld = _matrix(src)
    codes, scales = out if out is not None else (_u8((rows, cols // 2), src.device), _u8((rows, cols // 32), src.device))
    rc = lib().mx_quantize(_ptr(src), _src_dtype(src), rows, cols, ld, _ptr(codes), _ptr(scales),
                           round, scale_mode, seed, tensor_id, index_base, _stream(stream))
    _check("mx_quantize", rc)
    return codes, scales


def mx_quantize_e3m0(src, round=ROUND_RTN, scale_mode=SCALE_TRUNCFREE, seed=0, tensor_id=0, index_base=0,
                     out=None, stream=None):
    """mx_quantize with E3M0 elements (the format ablation's other 4-bit format); same packed layout."""
    rows, cols, ld = _matrix(src)
    codes, scales = out if out is not None else (_u8((rows, cols // 2), src.device), _u8((rows, cols // 32), src.device))
    rc = lib().mx_quantize_e3m0(_ptr(src), _src_dtype(src), rows, cols, ld, _ptr(codes), _ptr(scales),
                                round, scale_mode, seed, tensor_id, index_base, _stream(stream))
    _check("mx_quantize_e3m0", rc)
    return codes, scales


def mx_dequantize_e3m0(codes, scales, stream=None):
    rows, cols = codes.shape[0], codes.shape[1] * 2
    out = torch.empty((rows, cols), dtype=torch.float32, device=codes.device)
    rc = lib().mx_dequantize_e3m0(_ptr(codes), _ptr(scales), rows, cols, _ptr(out), _stream(stream))
    _check("mx_dequantize_e3m0", rc)
    return out


def mx_quantize_transposed(src, round_t=ROUND_SR, tensor_id_t=0, pre_quant=1, want_row=True,
                           round_row=ROUND_RTN, tensor_id_row=0, row_in=None,
                           scale_mode=SCALE_TRUNCFREE, seed=0, index_base=0, out=None, stream=None,
                           shape=None):
    """32x1 groups stored transposed, optionally fused with the 1x32 quantizer.

    Returns (codes_t[cols, rows/2], scales_t[cols, rows/32], codes_row, scales_row);
    the last two are None unless want_row.  With row_in=(codes, scales) the given
    row result is re-quantized and src may be None (pass shape=(rows, cols)).
    seed: an int, or a one-element int64 device tensor read by the kernel when it runs.
    """
    if src is not None:
        rows, cols, ld = _matrix(src)
        dtype, device = _src_dtype(src), src.device
    else:
        rows, cols = shape
        ld, dtype, device = cols, DTYPE_F32, row_in[0].device
    if out is not None:
        codes_t, scales_t, codes_row, scales_row = out
    else:
        codes_t, scales_t = _u8((cols, rows // 2), device), _u8((cols, rows // 32), device)
        codes_row = scales_row = None
        if want_row:
            codes_row, scales_row = _u8((rows, cols // 2), device), _u8((rows, cols // 32), device)
    if torch.is_tensor(seed):
        # a seed in device memory travels through the batched entry point (one request)
        job = {"out": (codes_t, scales_t, codes_row, scales_row), "tensor_id_t": tensor_id_t, "tensor_id_row": tensor_id_row,
               "pre_quant": pre_quant, "seed": seed, "index_base": index_base}
        job.update({"src": src} if src is not None else {"row_in": row_in, "shape": (rows, cols)})
        mx_quantize_transposed_batch([job], round_t, round_row, scale_mode, stream)
        return codes_t, scales_t, codes_row, scales_row
    rc_in, rs_in = row_in if row_in is not None else (None, None)
    rc = lib().mx_quantize_transposed(_ptr(src), dtype, rows, cols, ld, _ptr(codes_t), _ptr(scales_t),
                                      round_t, tensor_id_t, pre_quant, _ptr(codes_row), _ptr(scales_row),
                                      round_row, tensor_id_row, _ptr(rc_in), _ptr(rs_in),
                                      scale_mode, seed, index_base, _stream(stream))
    _check("mx_quantize_transposed", rc)
    return codes_t, scales_t, codes_row, scales_row


def mx_quantize_transposed_batch(jobs, round_t=ROUND_SR, round_row=ROUND_RTN, scale_mode=SCALE_TRUNCFREE, stream=None):
    """Several transposed quantizations in one launch.  jobs: list of dicts with the keys
    src, out=(codes_t, scales_t, codes_row, scales_row) and optionally tensor_id_t, tensor_id_row,
    pre_quant (1), seed (0), index_base (0), col_sums (a float32 tensor of `cols` values that receives the
    column sums of src; col_sum_workspace optional); the roundings and the scale rule are shared.
    Instead of src a job may give row_in=(codes, scales) and shape=(rows, cols).  seed may be a
    one-element int64 device tensor: the kernel then reads the seed from it when it runs
    (seed_dev of the C ABI), which is what a launch recorded into a graph needs."""
    arr = (_TransposedJob * len(jobs))()
    keep = []                                      # scratch made here lives until the launch is enqueued
    for j, job in zip(arr, jobs):
        src = job.get("src")
        codes_t, scales_t, codes_row, scales_row = job["out"]
        if src is not None:
            rows, cols, ld = _matrix(src)
            j.src, j.dtype, j.rows, j.cols, j.ld = src.data_ptr(), _src_dtype(src), rows, cols, ld
            j.row_codes_in = j.row_scales_in = None
        else:
            rows, cols = job["shape"]
            j.src, j.dtype, j.rows, j.cols, j.ld = None, DTYPE_F32, rows, cols, cols
            j.row_codes_in, j.row_scales_in = job["row_in"][0].data_ptr(), job["row_in"][1].data_ptr()
        j.codes_t, j.scales_t = codes_t.data_ptr(), scales_t.data_ptr()
        j.codes_row = codes_row.data_ptr() if codes_row is not None else None
        j.scales_row = scales_row.data_ptr() if scales_row is not None else None
        j.tensor_id_t, j.tensor_id_row = job.get("tensor_id_t", 0), job.get("tensor_id_row", 0)
        j.pre_quant, j.index_base = job.get("pre_quant", 1), job.get("index_base", 0)
        seed = job.get("seed", 0)
        if torch.is_tensor(seed):
            if seed.dtype != torch.int64 or seed.numel() != 1 or not seed.is_cuda:
                raise ValueError("a device seed is a one-element int64 tensor on the GPU")
            j.seed, j.seed_dev = 0, seed.data_ptr()
        else:
            j.seed, j.seed_dev = seed, None
        col_sums = job.get("col_sums")
        j.col_sums = j.col_sum_workspace = None
        if col_sums is not None:
            if col_sums.dtype != torch.float32 or not col_sums.is_contiguous() or col_sums.numel() != cols:
                raise ValueError("col_sums must be a contiguous float32 tensor of `cols` values")
            scratch = job.get("col_sum_workspace")
            need = int(lib().mx_column_sum_workspace_bytes(rows, cols))
            if scratch is None or scratch.numel() * scratch.element_size() < need:
                scratch = torch.empty(need // 4, dtype=torch.float32, device=col_sums.device)
            keep.append(scratch)
            j.col_sums, j.col_sum_workspace = col_sums.data_ptr(), scratch.data_ptr()
    rc = lib().mx_quantize_transposed_batch(arr, len(jobs), round_t, round_row, scale_mode, _stream(stream))
    _check("mx_quantize_transposed_batch", rc)


def mx_linear_workspace_bytes(which, N, C, D):
    return int(lib().mx_linear_workspace_bytes(which, N, C, D))


def _linear(name, which, a, a_s, b, b_s, N, C, D, out_shape, out, out_dtype, workspace, stream):
    device = a.device
    if out is None:
        out = torch.empty(out_shape, dtype=out_dtype, device=device)
    need = mx_linear_workspace_bytes(which, N, C, D)
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=device)
    wbytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = getattr(lib(), name)(_ptr(a), _ptr(a_s), _ptr(b), _ptr(b_s), N, C, D,
                              _ptr(out), _src_dtype(out), out.stride(0), _ptr(workspace), wbytes,
                              _stream(stream))
    _check(name, rc)
    return out


def mx_linear_fwd(xq, xs, wq, ws, out=None, out_dtype=torch.float32, workspace=None, stream=None):
    """Y[N, C] = Q1(X) . Q2(W)^T from packed operands xq[N, D/2], wq[C, D/2]."""
    N, D, C = xq.shape[0], xq.shape[1] * 2, wq.shape[0]
    return _linear("mx_linear_fwd", GEMM_FWD, xq, xs, wq, ws, N, C, D, (N, C), out, out_dtype, workspace, stream)


def mx_linear_fwd_bias(xq, xs, wq, ws, bias, out=None, out_dtype=torch.float32, workspace=None, stream=None):
    """Y[N, C] = Q1(X) . Q2(W)^T + bias, the bias (float32, C values) added in the product's output stage."""
    N, D, C = xq.shape[0], xq.shape[1] * 2, wq.shape[0]
    if bias.dtype != torch.float32 or not bias.is_contiguous() or bias.numel() != C:
        raise ValueError("bias must be a contiguous float32 tensor of C values")
    if out is None:
        out = torch.empty((N, C), dtype=out_dtype, device=xq.device)
    need = mx_linear_workspace_bytes(GEMM_FWD, N, C, D)
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=xq.device)
    wbytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = lib().mx_linear_fwd_bias(_ptr(xq), _ptr(xs), _ptr(wq), _ptr(ws), N, C, D, _ptr(bias),
                                  _ptr(out), _src_dtype(out), out.stride(0), _ptr(workspace), wbytes, _stream(stream))
    _check("mx_linear_fwd_bias", rc)
    return out


def mx_linear_fwd_gelu_quant(xq, xs, wq, ws, bias, out=None, out_dtype=torch.bfloat16, scale_mode=SCALE_TRUNCFREE,
                             quant_out=None, stream=None):
    """fc1 of an MLP with GELU and the next layer's forward quantizer in the product's output stage.
    Returns (P[N, C] pre-activation with bias, aq[N, C/2], as[N, C/32])."""
    N, D, C = xq.shape[0], xq.shape[1] * 2, wq.shape[0]
    if bias.dtype != torch.float32 or not bias.is_contiguous() or bias.numel() != C:
        raise ValueError("bias must be a contiguous float32 tensor of C values")
    if out is None:
        out = torch.empty((N, C), dtype=out_dtype, device=xq.device)
    aq, as_ = quant_out if quant_out is not None else (_u8((N, C // 2), xq.device), _u8((N, C // 32), xq.device))
    rc = lib().mx_linear_fwd_gelu_quant(_ptr(xq), _ptr(xs), _ptr(wq), _ptr(ws), N, C, D, _ptr(bias),
                                        _ptr(out), _src_dtype(out), out.stride(0), _ptr(aq), _ptr(as_), scale_mode,
                                        _stream(stream))
    _check("mx_linear_fwd_gelu_quant", rc)
    return out, aq, as_


def mx_linear_bwd_dx(dyq, dys, wtq, wts, out=None, out_dtype=torch.float32, workspace=None, stream=None):
    """dX[N, D] from dyq[N, C/2] and the transposed-quantized weight wtq[D, C/2]."""
    N, C, D = dyq.shape[0], dyq.shape[1] * 2, wtq.shape[0]
    return _linear("mx_linear_bwd_dx", GEMM_BWD_DX, dyq, dys, wtq, wts, N, C, D, (N, D), out, out_dtype, workspace, stream)


def mx_linear_bwd_dw(dytq, dyts, xtq, xts, out=None, out_dtype=torch.float32, workspace=None, stream=None):
    """dW[C, D] from dytq[C, N/2] and xtq[D, N/2]."""
    C, N, D = dytq.shape[0], dytq.shape[1] * 2, xtq.shape[0]
    return _linear("mx_linear_bwd_dw", GEMM_BWD_DW, dytq, dyts, xtq, xts, N, C, D, (C, D), out, out_dtype, workspace, stream)


NOALLOC_MAX_WORKSPACE_BYTES = 64 << 20


def mx_linear_bwd_dw_noalloc(dytq, dyts, xtq, xts, out, stream=None):
    """dW[C, D] into the caller's `out`, the K-split partials in the library's own device array: the
    call allocates nothing (so `out` is required)."""
    C, N, D = dytq.shape[0], dytq.shape[1] * 2, xtq.shape[0]
    if tuple(out.shape) != (C, D) or out.stride(1) != 1:
        raise ValueError("out must be [C, D] with unit column stride")
    rc = lib().mx_linear_bwd_dw_noalloc(_ptr(dytq), _ptr(dyts), _ptr(xtq), _ptr(xts), N, C, D,
                                        _ptr(out), _src_dtype(out), out.stride(0), _stream(stream))
    _check("mx_linear_bwd_dw_noalloc", rc)
    return out


def mx_ema_weight_quant(w, w_ema, beta=0.998, update_ema=1, scale_mode=SCALE_TRUNCFREE, out=None, stream=None):
    """Q-EMA; w_ema (float32, same shape and strides as w) is updated in place."""
    rows, cols, ld = _matrix(w)
    if w_ema.dtype != torch.float32 or w_ema.shape != w.shape or w_ema.stride() != w.stride():
        raise ValueError("w_ema must be float32 with the shape and strides of w")
    codes, scales = out if out is not None else (_u8((rows, cols // 2), w.device), _u8((rows, cols // 32), w.device))
    rc = lib().mx_ema_weight_quant(_ptr(w), _src_dtype(w), _ptr(w_ema), beta, update_ema, rows, cols, ld,
                                   _ptr(codes), _ptr(scales), scale_mode, _stream(stream))
    _check("mx_ema_weight_quant", rc)
    return codes, scales


class OscillationState:
    """Device buffers of one weight's detection window (Sec. 6.1)."""

    def __init__(self, rows, cols, device="cuda"):
        f = lambda: torch.empty((rows, cols), dtype=torch.float32, device=device)
        self.w_prev, self.dist_w, self.dist_q = f(), f(), f()
        self.codes_prev = _u8((rows, cols // 2), device)
        self.scales_prev = _u8((rows, cols // 32), device)
        self.started = False


def mx_oscillation_accumulate(w, codes, scales, state, init=None, stream=None):
    """One step of dist_W / dist_Q; init defaults to True on the state's first use."""
    rows, cols, ld = _matrix(w)
    if init is None:
        init = not state.started
    rc = lib().mx_oscillation_accumulate(_ptr(w), _src_dtype(w), rows, cols, ld, _ptr(codes), _ptr(scales),
                                         _ptr(state.w_prev), _ptr(state.codes_prev), _ptr(state.scales_prev),
                                         _ptr(state.dist_w), _ptr(state.dist_q), int(bool(init)), _stream(stream))
    _check("mx_oscillation_accumulate", rc)
    state.started = True
    return state


def mx_ramping_factor(dist_w, dist_q, k1=16.0, k2=5, n_max=16, out=None, stream=None):
    """N_w of Algorithm 2 per element (int32, shape of dist_w)."""
    if dist_w.dtype != torch.float32 or dist_q.dtype != torch.float32 or not dist_w.is_contiguous() or not dist_q.is_contiguous():
        raise ValueError("dist_w and dist_q must be contiguous float32 tensors")
    if out is None:
        out = torch.empty(dist_w.shape, dtype=torch.int32, device=dist_w.device)
    rc = lib().mx_ramping_factor(_ptr(dist_w), _ptr(dist_q), dist_w.numel(), float(k1), int(k2), int(n_max),
                                 _ptr(out), _stream(stream))
    _check("mx_ramping_factor", rc)
    return out


class RampingAdamwState:
    """Device state of Q-Ramping's customised AdamW for one weight: the two moments, the per-element
    update counts, and (ramping=True) the per-element gradient sums and their step counts."""

    def __init__(self, shape, device="cuda", ramping=True):
        self.shape = tuple(shape)
        z = lambda dt: torch.zeros(self.shape, dtype=dt, device=device)
        self.m, self.v, self.updates = z(torch.float32), z(torch.float32), z(torch.int32)
        self.g_acc = z(torch.float32) if ramping else None
        self.acc_steps = z(torch.int32) if ramping else None


def mx_ramping_adamw_step(w, grad, state, factor=None, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8,
                          weight_decay=0.01, stream=None):
    """One step of Algorithm 2's optimizer on the master weight w (float32, contiguous, in place).
    factor: int32 tensor from mx_ramping_factor, or None for plain AdamW."""
    if w.dtype != torch.float32 or not w.is_contiguous() or not grad.is_contiguous():
        raise ValueError("w must be contiguous float32, grad contiguous")
    if tuple(w.shape) != state.shape or grad.shape != w.shape:
        raise ValueError("shape mismatch")
    if factor is not None:
        if state.g_acc is None:
            raise ValueError("state was made without ramping")
        if factor.dtype != torch.int32 or not factor.is_contiguous() or factor.shape != w.shape:
            raise ValueError("factor must be a contiguous int32 tensor of w's shape")
    rc = lib().mx_ramping_adamw_step(_ptr(w), _ptr(grad), _src_dtype(grad), w.numel(), _ptr(state.m), _ptr(state.v),
                                     _ptr(state.updates), _ptr(factor),
                                     _ptr(state.g_acc if factor is not None else None),
                                     _ptr(state.acc_steps if factor is not None else None),
                                     float(lr), float(beta1), float(beta2), float(eps), float(weight_decay),
                                     _stream(stream))
    _check("mx_ramping_adamw_step", rc)
    return w


def mx_quant_confidence(w, scale_mode=SCALE_TRUNCFREE, conf=True, hist=None, stream=None):
    """Quantization confidence of Sec. 4.2.  conf=True returns the per-element confidences
    (float32, shape of w); hist (int64 tensor of `bins` counters) is added to if given.
    Returns (conf or None, hist or None)."""
    rows, cols = w.shape
    out = torch.empty((rows, cols), dtype=torch.float32, device=w.device) if conf else None
    bins = 0
    if hist is not None:
        if hist.dtype != torch.int64 or not hist.is_contiguous():
            raise ValueError("hist must be a contiguous int64 tensor")
        bins = hist.numel()
    rc = lib().mx_quant_confidence(_ptr(w), _src_dtype(w), rows, cols, w.stride(0), int(scale_mode),
                                   _ptr(out), _ptr(hist), bins, _stream(stream))
    _check("mx_quant_confidence", rc)
    return out, hist


class RateOfChangeState:
    """Device state of the rate of change of one tensor (Sec. 4.1): the previous tensor (FP32),
    the reduction scratch and the three result doubles (term, sum of terms, number of terms)."""

    def __init__(self, rows, cols, device="cuda"):
        self.rows, self.cols = rows, cols
        self.x_prev = torch.empty((rows, cols), dtype=torch.float32, device=device)
        self.workspace = torch.empty(lib().mx_rate_of_change_workspace_bytes(), dtype=torch.uint8, device=device)
        self.result = torch.zeros(3, dtype=torch.float64, device=device)
        self.started = False

    def rate(self):
        """r(X) over the terms since the window opened (synchronizes)."""
        _, total, count = self.result.tolist()
        return total / count if count else 0.0


def mx_rate_of_change_step(x, state, init=None, stream=None):
    """Adds ||x - x_prev||_F / ||x_prev||_F to the state's running sum, then x_prev <- x.
    init=True (default on first use) opens a window instead."""
    rows, cols = x.shape
    if (rows, cols) != (state.rows, state.cols):
        raise ValueError("state was made for another shape")
    if init is None:
        init = not state.started
    rc = lib().mx_rate_of_change_step(_ptr(x), _src_dtype(x), rows, cols, x.stride(0), _ptr(state.x_prev),
                                      1 if init else 0, _ptr(state.workspace), state.workspace.numel(),
                                      _ptr(state.result), _stream(stream))
    _check("mx_rate_of_change_step", rc)
    state.started = True
    return state


def mx_dequantize(codes, scales, stream=None):
    rows, cols = codes.shape[0], codes.shape[1] * 2
    out = torch.empty((rows, cols), dtype=torch.float32, device=codes.device)
    rc = lib().mx_dequantize(_ptr(codes), _ptr(scales), rows, cols, _ptr(out), _stream(stream))
    _check("mx_dequantize", rc)
    return out


def mx_calibration_copy(dst, src, stream=None):
    """Plain copy kernel (known HBM traffic) for scaling profiler byte counters."""
    nbytes = src.numel() * src.element_size()
    rc = lib().mx_calibration_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream))
    _check("mx_calibration_copy", rc)
    return dst


CALIBRATION_MFMA_OPERAND_BYTES = 98304


def mx_calibration_mfma(operands, workgroups, iterations, sink=None, stream=None):
    """Register-resident loop of the products' MFMA on the given operand bytes (uint8, at least
    CALIBRATION_MFMA_OPERAND_BYTES); returns the number of flops the launch performs."""
    if operands.dtype != torch.uint8 or operands.numel() < CALIBRATION_MFMA_OPERAND_BYTES or not operands.is_contiguous():
        raise ValueError("operands must be a contiguous uint8 tensor of at least %d bytes" % CALIBRATION_MFMA_OPERAND_BYTES)
    if sink is None:
        sink = torch.empty(workgroups * 512, dtype=torch.float32, device=operands.device)
    rc = lib().mx_calibration_mfma(_ptr(operands), workgroups, iterations, _ptr(sink), _stream(stream))
    _check("mx_calibration_mfma", rc)
    return workgroups * 8 * iterations * 16 * 2.0 * 32 * 32 * 64
