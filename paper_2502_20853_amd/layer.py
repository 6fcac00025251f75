"""One forward + backward pass of the MXFP4 linear layer (Eqs. 3-5, Sec. 3.3),
expressed as calls of the C ABI with preallocated buffers.  Plumbing only."""
import torch

from . import binding as B

# tensor ids of the six quantizers, numbered as in Eqs. 3-5
Q1, Q2, Q3, Q4, Q5, Q6 = 1, 2, 3, 4, 5, 6


class MxLinearStep:
    """Buffers and call sequence for X[N, D], W[C, D], dY[N, C].

    forward():  Q1/Q6 of X in one pass (row codes for Eq. 3, transposed double-quantized
                codes kept for Eq. 5), Q2/Q4 of W likewise, then Y.
    backward(): Q3/Q5 of dY in one pass, then dX (Eq. 4) and dW (Eq. 5).
    With qema=True the weight's row codes come from mx_ema_weight_quant and Q4
    re-quantizes those.
    seed: an int, or a one-element int64 device tensor that the quantizers read when they run.
    With the latter the whole pass can be recorded into a graph (the library allocates nothing
    and synchronizes nothing) and each replay rounds with the seed the tensor then holds.
    """

    def __init__(self, N, D, C, device="cuda", out_dtype=torch.bfloat16, dw_dtype=torch.float32,
                 qema=False, beta=0.998, scale_mode=B.SCALE_TRUNCFREE):
        if N % 32 or D % 32 or C % 32:
            raise ValueError("N, D and C must be multiples of 32 (each is a contraction dimension)")
        self.N, self.D, self.C = N, D, C
        self.qema, self.beta, self.scale_mode = qema, beta, scale_mode
        u8 = lambda *s: torch.empty(s, dtype=torch.uint8, device=device)
        self.xq, self.xs, self.xtq, self.xts = u8(N, D // 2), u8(N, D // 32), u8(D, N // 2), u8(D, N // 32)
        self.wq, self.ws, self.wtq, self.wts = u8(C, D // 2), u8(C, D // 32), u8(D, C // 2), u8(D, C // 32)
        self.dyq, self.dys, self.dytq, self.dyts = u8(N, C // 2), u8(N, C // 32), u8(C, N // 2), u8(C, N // 32)
        self.y = torch.empty((N, C), dtype=out_dtype, device=device)
        self.dx = torch.empty((N, D), dtype=out_dtype, device=device)
        self.dw = torch.empty((C, D), dtype=dw_dtype, device=device)
        need = max(B.mx_linear_workspace_bytes(w, N, C, D) for w in (B.GEMM_FWD, B.GEMM_BWD_DX, B.GEMM_BWD_DW))
        self.workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
        self.w_ema = None

    def quantize_weight(self, W, seed, update_ema=1):
        if self.qema:
            if self.w_ema is None:
                self.w_ema = torch.empty(W.shape, dtype=torch.float32, device=W.device)
                update_ema = 2
            B.mx_ema_weight_quant(W, self.w_ema, self.beta, update_ema, self.scale_mode, out=(self.wq, self.ws))
            B.mx_quantize_transposed(None, B.ROUND_SR, Q4, 1, False, row_in=(self.wq, self.ws),
                                     scale_mode=self.scale_mode, seed=seed, shape=(self.C, self.D),
                                     out=(self.wtq, self.wts, None, None))
        else:
            B.mx_quantize_transposed(W, B.ROUND_SR, Q4, 1, True, B.ROUND_RTN, Q2, scale_mode=self.scale_mode,
                                     seed=seed, out=(self.wtq, self.wts, self.wq, self.ws))

    def quantize_inputs(self, X, W, seed):
        """Q1/Q6 of X and Q2/Q4 of W: one launch when both are the same kind of source, else two."""
        if not self.qema and X.dtype == W.dtype:
            B.mx_quantize_transposed_batch(
                [{"src": X, "out": (self.xtq, self.xts, self.xq, self.xs), "tensor_id_t": Q6, "tensor_id_row": Q1, "seed": seed},
                 {"src": W, "out": (self.wtq, self.wts, self.wq, self.ws), "tensor_id_t": Q4, "tensor_id_row": Q2, "seed": seed}],
                B.ROUND_SR, B.ROUND_RTN, self.scale_mode)
        else:
            B.mx_quantize_transposed(X, B.ROUND_SR, Q6, 1, True, B.ROUND_RTN, Q1, scale_mode=self.scale_mode,
                                     seed=seed, out=(self.xtq, self.xts, self.xq, self.xs))
            self.quantize_weight(W, seed)

    def forward(self, X, W, seed):
        self.quantize_inputs(X, W, seed)
        return B.mx_linear_fwd(self.xq, self.xs, self.wq, self.ws, out=self.y, workspace=self.workspace)

    def backward(self, dY, seed):
        B.mx_quantize_transposed(dY, B.ROUND_SR, Q5, 0, True, B.ROUND_SR, Q3, scale_mode=self.scale_mode,
                                 seed=seed, out=(self.dytq, self.dyts, self.dyq, self.dys))
        B.mx_linear_bwd_dx(self.dyq, self.dys, self.wtq, self.wts, out=self.dx, workspace=self.workspace)
        B.mx_linear_bwd_dw(self.dytq, self.dyts, self.xtq, self.xts, out=self.dw, workspace=self.workspace)
        return self.dx, self.dw

    def step_two_streams(self, X, W, dY, seed, side, dw_workspace=None):
        """forward() + backward() with the launches spread over two streams: the current stream carries
        quant X -> forward product -> dX product, `side` carries quant W -> quant dY -> dW product; events
        express the data dependencies (the forward product needs the weight codes, dX the gradient codes,
        dW the transposed activation codes).  The sparsely filled last round of one kernel then overlaps the
        next kernel.  Same calls, same results as forward() and backward() (the library holds no state).
        dw_workspace: the dW product's own K-split workspace (it may run while dX uses self.workspace).
        When it returns, the current stream waits for `side`."""
        main = torch.cuda.current_stream()
        if dw_workspace is None:
            if getattr(self, "_dw_workspace", None) is None:
                self._dw_workspace = torch.empty_like(self.workspace)
            dw_workspace = self._dw_workspace
        fork, w_done, dy_done, x_done, join = (torch.cuda.Event() for _ in range(5))
        fork.record(main)
        side.wait_event(fork)                          # the layer's inputs are ready on the current stream
        with torch.cuda.stream(side):
            self.quantize_weight(W, seed)
            w_done.record()
            B.mx_quantize_transposed(dY, B.ROUND_SR, Q5, 0, True, B.ROUND_SR, Q3, scale_mode=self.scale_mode,
                                     seed=seed, out=(self.dytq, self.dyts, self.dyq, self.dys))
            dy_done.record()
        B.mx_quantize_transposed(X, B.ROUND_SR, Q6, 1, True, B.ROUND_RTN, Q1, scale_mode=self.scale_mode,
                                 seed=seed, out=(self.xtq, self.xts, self.xq, self.xs))
        x_done.record(main)
        main.wait_event(w_done)
        B.mx_linear_fwd(self.xq, self.xs, self.wq, self.ws, out=self.y, workspace=self.workspace)
        main.wait_event(dy_done)
        B.mx_linear_bwd_dx(self.dyq, self.dys, self.wtq, self.wts, out=self.dx, workspace=self.workspace)
        with torch.cuda.stream(side):
            side.wait_event(x_done)
            B.mx_linear_bwd_dw(self.dytq, self.dyts, self.xtq, self.xts, out=self.dw, workspace=dw_workspace)
            join.record()
        main.wait_event(join)
        return self.y, self.dx, self.dw
