"""Q-Ramping as a torch optimizer (Algorithm 2, Sec. 6): the schedule of the algorithm around the
library's kernels.  Plumbing only: every array operation is one of the C-ABI calls.

Every t_update steps a detection window of t0 steps opens.  Inside it the quantized weights take plain
AdamW steps (amplification factor 1 for every element) and the trajectory lengths dist_W, dist_Q of
Sec. 6.1 are accumulated from the weight before the window's first step to the weight after its last
one (t0 differences).  When the window closes, N_w = min(k2 * floor(R_w / k1) + 1, n_max) is computed
per element and used until the next window: an element then accumulates its gradient over N_w steps
and takes one AdamW step at N_w times the learning rate on the mean.  Parameters that are not
quantized take plain AdamW steps throughout.

Readings of the paper: the calibration steps of OscillationDetection are the training steps themselves;
w_Q is the forward quantizer's value of the master weight (1x32 groups along the input dimension, round
to nearest); gradients an element still holds when a window opens are applied at that step (their mean,
as one update).  t0 = 30 is the paper's value; t_update and n_max are not printed and must be chosen.
"""
import torch

from . import binding as B


def _view(cls, **fields):
    obj = cls.__new__(cls)
    for k, v in fields.items():
        setattr(obj, k, v)
    return obj


class QRampingAdamW(torch.optim.Optimizer):
    """quantized: the master weights of MXFP4 layers (float32, [out, in] with `in` a multiple of 32);
    others: every other parameter (float32).  step() reads p.grad of each."""

    def __init__(self, quantized, others=(), lr=1e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.01,
                 k1=16.0, k2=5, n_max=16, t0=30, t_update=1000, scale_mode=B.SCALE_TRUNCFREE):
        if not 0 < t0 < t_update:
            raise ValueError("need 0 < t0 < t_update (Algorithm 2: T0 << T_update)")
        if n_max < 1 or k2 < 0 or not k1 > 0:
            raise ValueError("need n_max >= 1, k2 >= 0, k1 > 0")
        groups = [{"params": list(quantized), "quantized": True}, {"params": list(others), "quantized": False}]
        for g in groups:
            for p in g["params"]:
                if p.dtype != torch.float32 or not p.is_contiguous():
                    raise ValueError("parameters must be contiguous float32 (master weights)")
                if p.numel() % 4:
                    raise ValueError("the optimizer kernel takes arrays whose length is a multiple of 4")
                if g["quantized"] and (p.dim() != 2 or p.shape[1] % 32):
                    raise ValueError("a quantized weight is [out, in] with `in` a multiple of 32")
        defaults = dict(lr=lr, betas=betas, eps=eps, weight_decay=weight_decay, k1=k1, k2=k2, n_max=n_max,
                        t0=t0, t_update=t_update, scale_mode=scale_mode, steps_done=0)
        super().__init__([g for g in groups if g["params"]], defaults)

    def _state(self, p, quantized):
        st = self.state[p]
        if not st:
            z = lambda dt: torch.zeros(p.shape, dtype=dt, device=p.device)
            st.update(m=z(torch.float32), v=z(torch.float32), updates=z(torch.int32))
            if quantized:
                rows, cols = p.shape
                u8 = lambda *s: torch.empty(s, dtype=torch.uint8, device=p.device)
                st.update(g_acc=z(torch.float32), acc_steps=z(torch.int32),
                          factor=torch.ones(p.shape, dtype=torch.int32, device=p.device),
                          ones=torch.ones(p.shape, dtype=torch.int32, device=p.device),
                          w_prev=z(torch.float32), dist_w=z(torch.float32), dist_q=z(torch.float32),
                          codes_prev=u8(rows, cols // 2), scales_prev=u8(rows, cols // 32),
                          codes=u8(rows, cols // 2), scales=u8(rows, cols // 32))
        return st

    @staticmethod
    def _track(p, st, scale_mode, init):
        B.mx_quantize(p.data, B.ROUND_RTN, scale_mode, out=(st["codes"], st["scales"]))
        osc = _view(B.OscillationState, w_prev=st["w_prev"], dist_w=st["dist_w"], dist_q=st["dist_q"],
                    codes_prev=st["codes_prev"], scales_prev=st["scales_prev"], started=True)
        B.mx_oscillation_accumulate(p.data, st["codes"], st["scales"], osc, init=init)

    def amplification_factors(self):
        """{parameter: N_w tensor in use} for the quantized weights (all ones before the first window closes)."""
        return {p: self.state[p]["factor"] for g in self.param_groups if g["quantized"] for p in g["params"] if self.state[p]}

    def load_state_dict(self, state_dict):
        """torch's loader converts every state tensor to its parameter's dtype; the integer arrays (update
        and step counts, factors, packed codes) are taken out before and put back unchanged after."""
        slim = {"state": {k: dict(v) for k, v in state_dict["state"].items()}, "param_groups": state_dict["param_groups"]}
        held = {k: {n: v.pop(n) for n in list(v) if torch.is_tensor(v[n]) and not v[n].is_floating_point()}
                for k, v in slim["state"].items()}
        super().load_state_dict(slim)
        params = [p for g in self.param_groups for p in g["params"]]
        for p in params:                                   # the kernels write in place: share nothing with the source
            for n, t in self.state[p].items():
                self.state[p][n] = t.clone()
        for k, tensors in held.items():
            for n, t in tensors.items():
                self.state[params[k]][n] = t.to(params[k].device).clone()

    @torch.no_grad()
    def step(self, closure=None):
        loss = None
        if closure is not None:
            with torch.enable_grad():
                loss = closure()
        for g in self.param_groups:
            phase = g["steps_done"] % g["t_update"]
            detecting = g["quantized"] and phase < g["t0"]
            for p in g["params"]:
                if p.grad is None and not detecting:
                    continue
                st = self._state(p, g["quantized"])
                adam = _view(B.RampingAdamwState, shape=tuple(p.shape), m=st["m"], v=st["v"], updates=st["updates"],
                             g_acc=st.get("g_acc"), acc_steps=st.get("acc_steps"))
                if detecting and phase == 0:
                    self._track(p, st, g["scale_mode"], True)          # the window's starting point w^0
                factor = None
                if g["quantized"]:
                    factor = st["ones"] if detecting else st["factor"]
                if p.grad is not None:                                 # a weight without a gradient stands still
                    B.mx_ramping_adamw_step(p.data, p.grad.contiguous(), adam, factor, g["lr"], g["betas"][0],
                                            g["betas"][1], g["eps"], g["weight_decay"])
                if detecting:
                    self._track(p, st, g["scale_mode"], False)
                    if phase == g["t0"] - 1:
                        B.mx_ramping_factor(st["dist_w"], st["dist_q"], g["k1"], g["k2"], g["n_max"], out=st["factor"])
            g["steps_done"] += 1
        return loss
