"""GPU tests of the autograd / nn.Module front end: what autograd returns for Y, dX, dW is what the
oracle computes for the same tensors, flows and seeds."""
import numpy as np
import pytest
import torch

from test_gpu_parity import check_product, dev, host, mx, oracle_layer  # noqa: F401  (mx: the fixture)

pytestmark = pytest.mark.gpu


def _padded(a, rows):
    out = np.zeros((rows, a.shape[1]), a.dtype)
    out[: a.shape[0]] = a
    return out


def _run_module(lin, X3, dY3):
    x = dev(X3).requires_grad_(True)
    y = lin(x)
    (y * dev(dY3)).sum().backward()                     # dL/dY = dY exactly
    return y.detach(), x.grad, lin.weight.grad


@pytest.mark.parametrize("flow", ["tetrajet", "microscaling"])
def test_module_forward_backward_matches_oracle(mx, orc, flow):
    """x[2, 100, 96] (200 tokens: padded to 224 with zero rows), 96 -> 160, with bias: Y, dX, dW from
    autograd against the oracle's products of the oracle's codes, for both flows of Sec. 3.3."""
    import mx_workloads as wl
    N, D, C, Np = 200, 96, 160, 224
    X, W, dY = wl.linear_layer(N, D, C, seed=2, outliers=2)
    lin = mx.MxLinear(D, C, bias=True, flow=flow, seed=3, layer_id=5)
    with torch.no_grad():
        lin.weight.copy_(dev(W))
        lin.bias.copy_(dev(np.linspace(-1, 1, C, dtype=np.float32)))
    y, dx, dw = _run_module(lin, X.reshape(2, 100, D), dY.reshape(2, 100, C))
    assert y.shape == (2, 100, C) and dx.shape == (2, 100, D) and dw.shape == (C, D)
    seed = ((3 << 16) | 5) << 32                        # first call of the module with seed 3 and layer id 5
    Xp, dYp = _padded(X, Np), _padded(dY, Np)
    if flow == "tetrajet":
        xt, wt, dy = oracle_layer(orc, Xp, W, dYp, seed=seed)
    else:                                               # Eqs. 6-7: deterministic, from the full-precision tensors
        xt = orc.quantize_transposed(Xp, round_t=0, tensor_id_t=6, pre_quant=0, round_row=0, tensor_id_row=1, seed=seed)
        wt = orc.quantize_transposed(W, round_t=0, tensor_id_t=4, pre_quant=0, round_row=0, tensor_id_row=2, seed=seed)
        dy = orc.quantize_transposed(dYp, round_t=0, tensor_id_t=5, pre_quant=0, round_row=0, tensor_id_row=3, seed=seed)
    bias = np.linspace(-1, 1, C, dtype=np.float32)
    y_nobias = torch.zeros((Np, C), device="cuda")
    y_nobias[:N] = y.reshape(N, C) - dev(bias)
    # subtracting the bias again costs one FP32 rounding of |y|: allow for it next to the product's 1e-5
    ref = orc.gemm_f64(xt[2], xt[3], wt[2], wt[3])
    absref = np.abs(orc.dequantize(xt[2], xt[3])) @ np.abs(orc.dequantize(wt[2], wt[3])).T
    err = np.abs(host(y_nobias).astype(np.float64) - ref)
    assert np.all(err <= 1e-5 * absref + 2.0 ** -22 * (np.abs(ref) + 1.0)), err.max()
    dxp = torch.zeros((Np, D), device="cuda")
    dxp[:N] = dx.reshape(N, D)
    ref_dx = orc.gemm_f64(dy[2], dy[3], wt[0], wt[1])
    assert np.all(ref_dx[N:] == 0.0)                    # zero gradient rows quantize to zero
    check_product(orc, dxp, dy[2], dy[3], wt[0], wt[1], "dX " + flow)
    check_product(orc, dw, dy[0], dy[1], xt[0], xt[1], "dW " + flow)
    want_db = dY.astype(np.float64).sum(0)
    assert np.allclose(host(lin.bias.grad), want_db, rtol=1e-5, atol=1e-5 * np.abs(dY).sum(0).max())
    # a second call draws new rounding streams (seed advances with the call count)
    y2, dx2, _ = _run_module(lin, X.reshape(2, 100, D), dY.reshape(2, 100, C))
    assert torch.equal(y2, y)                           # the forward quantizers are deterministic
    if flow == "tetrajet":
        assert not torch.equal(dx2, dx)
    else:
        assert torch.equal(dx2, dx)


def test_module_qema_and_bf16(mx, orc):
    """bf16 activations and weights, weight through Q-EMA: two training-mode forwards advance the
    moving average exactly as the oracle does, and Y is the product with the Q-EMA codes."""
    import mx_workloads as wl
    N, D, C = 256, 128, 96
    X, _, _ = wl.linear_layer(N, D, C, seed=6, dtype="bf16")
    lin = mx.MxLinear(D, C, bias=False, dtype=torch.bfloat16, qema=True, beta=0.99, seed=1)
    ema = None
    for t, W in enumerate(wl.weight_walk(C, D, seed=6, steps=1, sigma=5e-3)):
        W = wl.round_to_bf16(W)
        if ema is None:
            ema = np.zeros_like(W)
        wc, wsc = orc.ema_weight_quant(W, ema, beta=0.99, update_ema=2 if t == 0 else 1)
        with torch.no_grad():
            lin.weight.copy_(dev(W, "bf16"))
        y = lin(dev(X, "bf16"))
        assert np.array_equal(host(lin.w_ema), ema), t
    assert y.dtype == torch.bfloat16
    xq = orc.quantize(X)
    ref = orc.gemm_f64(xq[0], xq[1], wc, wsc)
    absref = np.abs(orc.dequantize(xq[0], xq[1])) @ np.abs(orc.dequantize(wc, wsc)).T
    err = np.abs(host(y.detach().float()).astype(np.float64) - ref)
    assert np.all(err <= 1e-5 * absref + 2.0 ** -8 * np.abs(ref))      # bf16 output rounding
    # evaluation mode leaves the moving average alone
    lin.eval()
    before = lin.w_ema.clone()
    lin(dev(X, "bf16"))
    assert torch.equal(before, lin.w_ema)


def test_module_trains_a_small_mlp(mx):
    """Two MXFP4 layers fit a random teacher: the loss must fall (a property, not a parity check --
    gradients that were wrong in sign, scale or transposition would not descend)."""
    torch.manual_seed(0)
    Din, H, Dout, N = 64, 128, 32, 512
    teacher = torch.randn(Din, Dout, device="cuda") / Din ** 0.5
    x = torch.randn(N, Din, device="cuda")
    target = torch.tanh(x @ teacher)
    net = torch.nn.Sequential(mx.MxLinear(Din, H, seed=1), torch.nn.GELU(), mx.MxLinear(H, Dout, seed=2))
    opt = torch.optim.AdamW(net.parameters(), lr=3e-3, weight_decay=0.0)
    losses = []
    for _ in range(60):
        opt.zero_grad()
        loss = torch.nn.functional.mse_loss(net(x), target)
        loss.backward()
        opt.step()
        losses.append(float(loss.detach()))
    assert losses[-1] < 0.5 * losses[0], (losses[0], losses[-1])


def test_module_device_seed_equals_host_seed_and_replays_in_a_graph(mx):
    """device_seed=True: the same Y, dX, dW as the host-side key, call for call (eagerly); and a whole
    forward + backward recorded into a graph gives, replay after replay, what the eager module gives on
    its next calls (new rounding numbers each time, so the gradients of two replays differ)."""
    import mx_workloads as wl
    N, D, C = 96, 64, 128
    X, W, dY = wl.linear_layer(N, D, C, seed=8)
    lins = [mx.MxLinear(D, C, bias=True, seed=0x9ABC, layer_id=0xDEF0, device_seed=ds) for ds in (False, True)]
    for lin in lins:
        with torch.no_grad():
            lin.weight.copy_(dev(W))
            lin.bias.copy_(dev(np.linspace(-2, 2, C, dtype=np.float32)))

    def eager(lin):
        x = dev(X).requires_grad_(True)
        lin.weight.grad = lin.bias.grad = None
        y = lin(x)
        (y * dev(dY)).sum().backward()
        return y.detach().clone(), x.grad.clone(), lin.weight.grad.clone(), lin.bias.grad.clone()

    for call in range(2):
        a, b = eager(lins[0]), eager(lins[1])
        for u, v, nm in zip(a, b, ("Y", "dX", "dW", "dbias")):
            assert torch.equal(u, v), (call, nm)
    # record call 3 of the device-seed module; replays are then calls 3, 4, 5 of the host-seed module
    lin = lins[1]
    xs = dev(X).requires_grad_(True)
    dys = dev(dY)
    lin.weight.grad = lin.bias.grad = None
    graph = torch.cuda.CUDAGraph()
    before = lin.seed_state.clone()
    with torch.cuda.graph(graph):
        ys = lin(xs)
        (ys * dys).sum().backward()
    lin.seed_state.copy_(before)                       # recording ran nothing: the key still names call 2
    seen = []
    for call in range(3):
        graph.replay()
        torch.cuda.synchronize()
        want = eager(lins[0])
        for u, v, nm in zip((ys, xs.grad, lin.weight.grad, lin.bias.grad), want, ("Y", "dX", "dW", "dbias")):
            assert torch.equal(u, v), (call, nm)
        seen.append(xs.grad.clone())
    assert not torch.equal(seen[0], seen[1]) and not torch.equal(seen[1], seen[2])


def test_layers_of_a_model_round_with_independent_streams(mx):
    """Two layers of the same shape built with default arguments, given the same weight, input and output
    gradient: the deterministic forward agrees bit for bit, the stochastically rounded backward does not
    (each layer's Philox key carries its own layer id, Sec. 3.4's independence)."""
    import mx_workloads as wl
    N, D, C = 96, 64, 128
    X, W, dY = wl.linear_layer(N, D, C, seed=12)
    a, b = mx.MxLinear(D, C, bias=False), mx.MxLinear(D, C, bias=False)
    assert a.layer_id != b.layer_id and a.key_high != b.key_high
    outs = []
    for lin in (a, b):
        with torch.no_grad():
            lin.weight.copy_(dev(W))
        outs.append(_run_module(lin, X, dY))
    assert torch.equal(outs[0][0], outs[1][0])
    assert not torch.equal(outs[0][1], outs[1][1]) and not torch.equal(outs[0][2], outs[1][2])


def test_device_seed_backward_uses_the_key_of_its_own_forward(mx):
    """Two forward calls before the first backward (micro-batches): with the key in device memory each
    backward still rounds with the key of its own forward, as the host-side key does."""
    import mx_workloads as wl
    N, D, C = 64, 64, 96
    X, W, dY = wl.linear_layer(N, D, C, seed=13)
    grads = []
    for ds in (False, True):
        lin = mx.MxLinear(D, C, bias=False, seed=4, layer_id=9, device_seed=ds)
        with torch.no_grad():
            lin.weight.copy_(dev(W))
        x1, x2 = dev(X).requires_grad_(True), dev(X).requires_grad_(True)
        y1, y2 = lin(x1), lin(x2)
        (y1 * dev(dY)).sum().backward()
        (y2 * dev(dY)).sum().backward()
        grads.append((x1.grad.clone(), x2.grad.clone()))
    assert torch.equal(grads[0][0], grads[1][0]) and torch.equal(grads[0][1], grads[1][1])
    assert not torch.equal(grads[0][0], grads[0][1])
