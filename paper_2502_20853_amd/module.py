"""torch.autograd / nn.Module front end of the MXFP4 linear layer: the forward and backward of Eqs. 3-5
(Sec. 3.3) as calls of the C ABI.  Plumbing only -- every quantizer and every product runs in the HIP
library; what is saved for the backward pass is the packed 4-bit operands, not the activations."""
import itertools

import torch

from . import binding as B
from .layer import Q1, Q2, Q3, Q4, Q5, Q6

TETRAJET, MICROSCALING = "tetrajet", "microscaling"

# Layers are numbered in the order they are constructed; the number goes into every layer's Philox key
# so that two layers never round with the same random numbers (see MxLinear).
_layer_ids = itertools.count()


def _pad_rows(t, rows):
    """t[N, K] with zero rows appended up to `rows` (a 32x1 group along the tokens must be whole; zero
    rows change no group maximum and add nothing to dW)."""
    if t.shape[0] == rows:
        return t
    out = t.new_zeros((rows, t.shape[1]))
    out[: t.shape[0]] = t
    return out


class _MxLinearFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x2d, weight, bias, mod, seed):
        N, D = x2d.shape
        C = weight.shape[0]
        Np = (N + 31) // 32 * 32
        x2d = _pad_rows(x2d.contiguous(), Np)
        tetra = mod.flow == TETRAJET
        rnd_t = B.ROUND_SR if tetra else B.ROUND_RTN           # Eqs. 4-5 vs Eqs. 6-7
        pre = 1 if tetra else 0
        if not mod.qema and x2d.dtype == weight.dtype:
            # activation and weight in one launch
            u8 = lambda *shape: torch.empty(shape, dtype=torch.uint8, device=x2d.device)
            xtq, xts, xq, xs = u8(D, Np // 2), u8(D, Np // 32), u8(Np, D // 2), u8(Np, D // 32)
            wtq, wts, wq, ws = u8(D, C // 2), u8(D, C // 32), u8(C, D // 2), u8(C, D // 32)
            B.mx_quantize_transposed_batch(
                [{"src": x2d, "out": (xtq, xts, xq, xs), "tensor_id_t": Q6, "tensor_id_row": Q1, "pre_quant": pre, "seed": seed},
                 {"src": weight.detach(), "out": (wtq, wts, wq, ws), "tensor_id_t": Q4, "tensor_id_row": Q2, "pre_quant": pre,
                  "seed": seed}], rnd_t, B.ROUND_RTN, mod.scale_mode)
        else:
            xtq, xts, xq, xs = B.mx_quantize_transposed(x2d, rnd_t, Q6, pre, True, B.ROUND_RTN, Q1,
                                                        scale_mode=mod.scale_mode, seed=seed)
            wq, ws, wtq, wts = mod._quantize_weight(weight, rnd_t, pre, seed)
        ws_fwd = mod._workspace(B.GEMM_FWD, Np, C, D)
        if bias is None:
            y = B.mx_linear_fwd(xq, xs, wq, ws, out_dtype=x2d.dtype, workspace=ws_fwd)
        else:                                              # added in the product's output stage
            y = B.mx_linear_fwd_bias(xq, xs, wq, ws, bias.detach().float().contiguous(), out_dtype=x2d.dtype,
                                     workspace=ws_fwd)
        ctx.save_for_backward(xtq, xts, wtq, wts)
        ctx.bias_dtype = None if bias is None else bias.dtype
        ctx.mod, ctx.seed, ctx.N, ctx.x_dtype, ctx.w_dtype = mod, seed, N, x2d.dtype, weight.dtype
        return y[:N]

    @staticmethod
    def backward(ctx, dy):
        xtq, xts, wtq, wts = ctx.saved_tensors
        mod, N = ctx.mod, ctx.N
        D, C, Np = xtq.shape[0], wtq.shape[1] * 2, xtq.shape[1] * 2
        dy = _pad_rows(dy.contiguous(), Np)
        rnd = B.ROUND_SR if mod.flow == TETRAJET else B.ROUND_RTN
        dbias = None
        if ctx.bias_dtype is not None and ctx.needs_input_grad[2]:
            # the bias gradient is the column sum of dY: taken by the quantizer from the values it loads
            # (the zero rows of the padding add nothing)
            u8 = lambda *shape: torch.empty(shape, dtype=torch.uint8, device=dy.device)
            dytq, dyts, dyq, dys = u8(C, Np // 2), u8(C, Np // 32), u8(Np, C // 2), u8(Np, C // 32)
            dbias = torch.empty(C, dtype=torch.float32, device=dy.device)
            B.mx_quantize_transposed_batch(
                [{"src": dy, "out": (dytq, dyts, dyq, dys), "tensor_id_t": Q5, "tensor_id_row": Q3, "pre_quant": 0,
                  "seed": ctx.seed, "col_sums": dbias}], rnd, rnd, mod.scale_mode)
            dbias = dbias.to(ctx.bias_dtype)
        else:
            dytq, dyts, dyq, dys = B.mx_quantize_transposed(dy, rnd, Q5, 0, True, rnd, Q3,
                                                            scale_mode=mod.scale_mode, seed=ctx.seed)
        dx = dw = None
        if ctx.needs_input_grad[0]:
            dx = B.mx_linear_bwd_dx(dyq, dys, wtq, wts, out_dtype=ctx.x_dtype,
                                    workspace=mod._workspace(B.GEMM_BWD_DX, Np, C, D))[:N]
        if ctx.needs_input_grad[1]:
            dw = B.mx_linear_bwd_dw(dytq, dyts, xtq, xts, out_dtype=torch.float32,
                                    workspace=mod._workspace(B.GEMM_BWD_DW, Np, C, D))
            if ctx.w_dtype != torch.float32:
                dw = dw.to(ctx.w_dtype)
        return dx, dw, dbias, None, None


class MxLinear(torch.nn.Module):
    """y = x W^T (+ bias) with the three products in MXFP4 (Eqs. 3-5).

    in_features and out_features must be multiples of 32; the token count (product of the leading
    dimensions of x) is padded with zero rows to a multiple of 32.  x and weight are float32 or
    bfloat16.  flow="tetrajet": deterministic forward quantizers, stochastic backward quantizers,
    double quantization (Sec. 3.3); flow="microscaling": Eqs. 6-7 (all deterministic, the backward
    operands quantized from the full-precision tensors).  qema=True takes the forward weight codes
    from Q-EMA (Sec. 5); the moving average advances once per training-mode forward.

    Stochastic rounding streams.  The 64-bit Philox key of a forward call and of its backward is
    (seed & 0xFFFF) << 48 | (layer_id & 0xFFFF) << 32 | number of forward calls so far.  layer_id
    defaults to the layer's position in the order of construction in this process, so the layers of a
    model draw independent numbers (the unbiasedness argument of Sec. 3.4 needs the rounding of dY in
    one layer to be independent of the rounding that produced it in the next); pass layer_id to fix
    it, e.g. to reproduce a run with a different construction order.  device_seed=True keeps the key in
    device memory and advances it with a kernel, so that a forward + backward recorded into a graph
    rounds with new numbers on every replay (same values as the host-side key, call for call); each
    forward call keeps its own copy of the key for its backward, so several forwards may precede the
    first backward (micro-batches, a module used twice).
    """

    def __init__(self, in_features, out_features, bias=True, device="cuda", dtype=torch.float32,
                 flow=TETRAJET, scale_mode=B.SCALE_TRUNCFREE, qema=False, beta=0.998, seed=0, device_seed=False,
                 layer_id=None):
        super().__init__()
        if in_features % 32 or out_features % 32:
            raise ValueError("in_features and out_features must be multiples of 32")
        if flow not in (TETRAJET, MICROSCALING):
            raise ValueError("flow must be 'tetrajet' or 'microscaling'")
        self.in_features, self.out_features = in_features, out_features
        self.flow, self.scale_mode, self.qema, self.beta, self.seed = flow, scale_mode, qema, beta, int(seed)
        self.weight = torch.nn.Parameter(torch.empty((out_features, in_features), device=device, dtype=dtype))
        self.bias = torch.nn.Parameter(torch.zeros(out_features, device=device, dtype=dtype)) if bias else None
        torch.nn.init.trunc_normal_(self.weight, std=0.02)
        self.register_buffer("w_ema", torch.zeros((out_features, in_features), device=device, dtype=torch.float32)
                             if qema else None)
        self.calls = 0                     # forward calls so far (host-side: reading it must not synchronize)
        self.layer_id = next(_layer_ids) if layer_id is None else int(layer_id)
        self.key_high = ((self.seed & 0xFFFF) << 16) | (self.layer_id & 0xFFFF)   # upper 32 bits of the Philox key
        start = ((self.key_high << 32) - 1) & 0xFFFFFFFFFFFFFFFF                 # one before the first key, as a 64-bit word
        self.register_buffer("seed_state", torch.tensor([start - (1 << 64) if start >> 63 else start], dtype=torch.int64,
                                                        device=device) if device_seed else None)
        self._ema_started = False
        self._ws = None

    def _workspace(self, which, N, C, D):
        need = B.mx_linear_workspace_bytes(which, N, C, D)
        if need == 0:
            return None
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.weight.device)
        return self._ws

    def _quantize_weight(self, weight, rnd_t, pre, seed):
        """Row codes (Q2, or Q-EMA) and transposed codes (Q4) of the weight."""
        if self.qema:
            update = 0
            if self.training:
                update = 1 if self._ema_started else 2
                self._ema_started = True
            elif not self._ema_started:
                update, self._ema_started = 2, True
            wq, ws = B.mx_ema_weight_quant(weight.detach(), self.w_ema, self.beta, update, self.scale_mode)
            if pre:
                wtq, wts, _, _ = B.mx_quantize_transposed(None, rnd_t, Q4, 1, False, row_in=(wq, ws),
                                                          scale_mode=self.scale_mode, seed=seed,
                                                          shape=tuple(weight.shape))
            else:
                wtq, wts, _, _ = B.mx_quantize_transposed(weight.detach(), rnd_t, Q4, 0, False,
                                                          scale_mode=self.scale_mode, seed=seed)
            return wq, ws, wtq, wts
        wtq, wts, wq, ws = B.mx_quantize_transposed(weight.detach(), rnd_t, Q4, pre, True, B.ROUND_RTN, Q2,
                                                    scale_mode=self.scale_mode, seed=seed)
        return wq, ws, wtq, wts

    def forward(self, x):
        lead = x.shape[:-1]
        x2d = x.reshape(-1, self.in_features)
        if self.seed_state is not None:
            # the word the kernels read: this call's own copy, which its backward pass reads too, so
            # that later forward calls (which advance seed_state) do not change it
            seed = self.seed_state.add_(1).clone()
        else:
            seed = (self.key_high << 32) + (self.calls & 0xFFFFFFFF)
        self.calls += 1
        y = _MxLinearFn.apply(x2d, self.weight, self.bias, self, seed)
        return y.reshape(*lead, self.out_features)
