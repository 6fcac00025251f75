"""GPU tests of the Q-Ramping optimizer front end (Algorithm 2): its schedule against the same
sequence of library calls written out step by step, the behaviour the algorithm is built for on a
weight that oscillates by construction, and plain AdamW where nothing oscillates.  The kernels it calls
are compared with the oracle in test_gpu_parity.py."""
import numpy as np
import pytest
import torch

from test_gpu_parity import dev, host, mx  # noqa: F401  (mx: the fixture)

pytestmark = pytest.mark.gpu


def _gradients(rows, cols, steps, seed, alternating):
    """Seeded gradients; the columns named in `alternating` change sign every step (weights pushed back
    and forth across whatever threshold they sit near)."""
    rng = np.random.default_rng(seed)
    g = 0.05 * rng.standard_normal((steps, rows, cols)).astype(np.float32)
    sign = np.where(np.arange(steps) % 2 == 0, 1.0, -1.0).astype(np.float32)
    g[:, :, alternating] = sign[:, None, None] * (1.0 + 0.01 * rng.standard_normal((1, rows, len(alternating)))).astype(np.float32)
    return g


def test_schedule_equals_the_calls_written_out(mx):
    """t0 = 4, t_update = 9 over 24 steps (three windows): weights, factors and optimizer state equal,
    bit for bit, those of the library calls issued by hand in the order Algorithm 2 gives."""
    B = mx.binding
    rows, cols, steps, t0, tu = 48, 96, 24, 4, 9
    k1, k2, nmax, lr = 2.0, 2, 8, 3e-3
    rng = np.random.default_rng(1)
    w0 = rng.standard_normal((rows, cols)).astype(np.float32)
    b0 = rng.standard_normal(cols).astype(np.float32)
    grads = _gradients(rows, cols, steps, 2, alternating=list(range(0, 32)))
    bgrads = 0.1 * rng.standard_normal((steps, cols)).astype(np.float32)

    w = torch.nn.Parameter(dev(w0))
    b = torch.nn.Parameter(dev(b0))
    opt = mx.QRampingAdamW([w], [b], lr=lr, k1=k1, k2=k2, n_max=nmax, t0=t0, t_update=tu, weight_decay=0.02)

    w_ref, b_ref = dev(w0), dev(b0)
    ad_w = B.RampingAdamwState((rows, cols), ramping=True)
    ad_b = B.RampingAdamwState((cols,), ramping=False)
    osc = B.OscillationState(rows, cols)
    ones = torch.ones((rows, cols), dtype=torch.int32, device="cuda")
    factor = ones.clone()
    seen = set()
    for t in range(steps):
        w.grad, b.grad = dev(grads[t]), dev(bgrads[t])
        opt.step()
        phase = t % tu
        if phase == 0:
            B.mx_oscillation_accumulate(w_ref, *B.mx_quantize(w_ref), osc, init=True)
        B.mx_ramping_adamw_step(w_ref, dev(grads[t]), ad_w, ones if phase < t0 else factor, lr=lr, weight_decay=0.02)
        B.mx_ramping_adamw_step(b_ref, dev(bgrads[t]), ad_b, None, lr=lr, weight_decay=0.02)
        if phase < t0:
            B.mx_oscillation_accumulate(w_ref, *B.mx_quantize(w_ref), osc, init=False)
            if phase == t0 - 1:
                factor = B.mx_ramping_factor(osc.dist_w, osc.dist_q, k1, k2, nmax)
        assert torch.equal(w.data, w_ref), t
        assert torch.equal(b.data, b_ref), t
        assert torch.equal(opt.amplification_factors()[w], factor), t
        seen.update(np.unique(host(factor)).tolist())
    st = opt.state[w]
    for name, ref in (("m", ad_w.m), ("v", ad_w.v), ("updates", ad_w.updates), ("g_acc", ad_w.g_acc), ("acc_steps", ad_w.acc_steps),
                      ("dist_w", osc.dist_w), ("dist_q", osc.dist_q)):
        assert torch.equal(st[name], ref), name
    assert min(seen) == 1 and max(seen) > 1           # the run did amplify some elements and left others alone


def test_oscillating_elements_are_amplified_and_stop_flipping(mx):
    """Weights placed next to a quantization threshold and pushed across it and back by a sign-alternating
    gradient (first moment all but switched off, so every step is about lr long) flip their quantized value every step under AdamW.  After the first window those elements (and only
    those) carry N_w > 1; with the mean of an alternating gradient near zero they then stay put, so
    dist_Q over a later stretch of steps falls to a fraction of what plain AdamW keeps producing."""
    B = mx.binding
    rows, cols, t0, tu, lr = 32, 64, 6, 40, 2e-2
    w0 = np.full((rows, cols), 0.4, np.float32)
    w0[:, 0::32] = 6.0                                 # group maximum 6 -> S = 1: thresholds at 0.25, 0.75, ...
    w0[:, 1:9] = 0.76                                  # eight elements per row next to the 0.5 | 1.0 threshold (0.75)
    grads = np.zeros((tu, rows, cols), np.float32)
    grads[:, :, 1:9] = np.where(np.arange(tu) % 2 == 0, 1.0, -1.0).astype(np.float32)[:, None, None]

    def run(ramping):
        w = torch.nn.Parameter(dev(w0))
        opt = mx.QRampingAdamW([w], lr=lr, betas=(1e-3, 0.999), k1=4.0, k2=3, n_max=16 if ramping else 1, t0=t0,
                               t_update=tu, weight_decay=0.0)
        osc = B.OscillationState(rows, cols)
        for t in range(tu):
            if t == t0:
                B.mx_oscillation_accumulate(w.data, *B.mx_quantize(w.data), osc, init=True)
            w.grad = dev(grads[t])
            opt.step()
            if t >= t0:
                B.mx_oscillation_accumulate(w.data, *B.mx_quantize(w.data), osc, init=False)
        return host(opt.amplification_factors()[w]), host(osc.dist_q)

    f_on, dq_on = run(True)
    f_off, dq_off = run(False)
    assert np.all(f_off == 1)
    assert np.all(f_on[:, 1:9] > 1) and np.all(np.delete(f_on, np.s_[1:9], axis=1) == 1)
    assert dq_off[:, 1:9].min() > 0                    # plain AdamW keeps flipping them
    assert dq_on[:, 1:9].sum() < 0.25 * dq_off[:, 1:9].sum()
    assert dq_on[:, 9:32].sum() == 0 and dq_off[:, 9:32].sum() == 0


def test_plain_adamw_when_nothing_oscillates(mx):
    """With n_max = 1 every element keeps factor 1: the optimizer is AdamW (against torch.optim.AdamW in
    FP64, to FP32 accuracy) for quantized and other parameters alike, across a window boundary."""
    rows, cols, steps = 40, 64, 25
    rng = np.random.default_rng(7)
    w0 = rng.standard_normal((rows, cols)).astype(np.float32)
    b0 = rng.standard_normal(rows).astype(np.float32)
    gw = rng.standard_normal((steps, rows, cols)).astype(np.float32)
    gb = rng.standard_normal((steps, rows)).astype(np.float32)
    w, b = torch.nn.Parameter(dev(w0)), torch.nn.Parameter(dev(b0))
    opt = mx.QRampingAdamW([w], [b], lr=1e-2, n_max=1, t0=3, t_update=10, weight_decay=0.05)
    wr = torch.nn.Parameter(torch.from_numpy(w0).double())
    br = torch.nn.Parameter(torch.from_numpy(b0).double())
    ref = torch.optim.AdamW([wr, br], lr=1e-2, weight_decay=0.05)
    for t in range(steps):
        w.grad, b.grad = dev(gw[t]), dev(gb[t])
        wr.grad, br.grad = torch.from_numpy(gw[t]).double(), torch.from_numpy(gb[t]).double()
        opt.step()
        ref.step()
    assert np.allclose(host(w.data), wr.detach().numpy(), rtol=2e-5, atol=2e-6)
    assert np.allclose(host(b.data), br.detach().numpy(), rtol=2e-5, atol=2e-6)
