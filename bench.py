"""Benchmark of the MXFP4 linear-layer hot path on one MI355X.

One step = forward + backward of the four linear layers of a ViT-B/16 block
(qkv, proj, fc1, fc2) at batch 256 (N = 50432 tokens): per layer the fused
row/transposed quantizers of X, W and dY and the three block-scaled FP4
products, all through the C ABI.  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP4_TFLOPS = 10100.0      # MI355X dense FP4/FP6 matrix peak
PEAK_HBM_GBS = 8000.0


class BoardPower:
    """Board power of GPU 0 from the amdgpu hwmon files (microwatts), sampled by a thread every 10 ms.
    Reading the files touches neither the HIP runtime nor the streams; where they are absent every
    figure is None."""

    def __init__(self):
        import glob
        self.path = self.cap_w = None
        for h in sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*")):
            for name in ("power1_input", "power1_average"):
                if self.path is None and os.path.exists(os.path.join(h, name)):
                    self.path = os.path.join(h, name)
            cap = os.path.join(h, "power1_cap")
            if self.cap_w is None and os.path.exists(cap):
                try:
                    self.cap_w = int(open(cap).read()) / 1e6
                except (OSError, ValueError):
                    pass
        self.samples, self._stop, self._thread = [], False, None

    def _read(self):
        try:
            return int(open(self.path).read()) / 1e6
        except (OSError, ValueError, TypeError):
            return None

    def start(self):
        import threading
        self.samples, self._stop = [], False

        def loop():
            while not self._stop:
                w = self._read()
                if w is not None:
                    self.samples.append((time.perf_counter(), w))
                time.sleep(0.01)
        if self.path is not None:
            self._thread = threading.Thread(target=loop, daemon=True)
            self._thread.start()

    def stop(self, since=None):
        """Mean watts of the samples taken after `since` (a perf_counter value), or None."""
        self._stop = True
        if self._thread is not None:
            self._thread.join()
            self._thread = None
        w = [x for (t, x) in self.samples if since is None or t >= since]
        return round(sum(w) / len(w), 1) if w else None

    def watts_of(self, fn, sync, seconds=0.4):
        """Mean board power while fn() is issued back to back for `seconds` (the first third is left out)."""
        if self.path is None:
            return None
        sync()
        self.start()
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < seconds:
            for _ in range(4):
                fn()
            sync()
        return self.stop(since=t0 + seconds / 3)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="vit_base_b256")
    ap.add_argument("--tokens", type=int, default=None, help="override N (tokens) of the workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=16384)
    ap.add_argument("--traffic-json", default=os.path.join(ROOT, "profiles", "gemm_traffic.json"),
                    help="HBM bytes per GEMM launch measured with rocprofv3 --pmc, if present")
    ap.add_argument("--event-every", type=int, default=5,
                    help="record the per-kernel HIP events on every n-th timed step (an event between two "
                         "launches costs about 3 us of idle chip, 5 %% of a step if every step carries them)")
    ap.add_argument("--no-other-schedule", action="store_true",
                    help="skip the comparison pass under the other stream schedule (for profiler runs: its "
                         "overlapped kernels would mix into the per-kernel statistics)")
    ap.add_argument("--streams", type=int, default=1, choices=(1, 2),
                    help="2: the timed steps without per-kernel events issue the weight / gradient quantizers and the dW "
                         "product on a second HIP stream (MxLinearStep.step_two_streams); once the chip is warm this "
                         "measures the same as one stream, which stays the default")
    ap.add_argument("--settle-ms", type=float, default=250.0,
                    help="untimed steps are run for this long before the W warm-up steps: after the idle time of input "
                         "generation the chip needs about 100 ms of load before its clocks settle (the first steps "
                         "run 5 %% slower), which W = 3..5 steps (7 ms) do not provide")
    ap.add_argument("--no-power", action="store_true",
                    help="skip the board-power loops after the timed region (for profiler runs: 0.4 s of back-to-back "
                         "launches per kernel family would swamp the per-kernel statistics)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference dispatch for scaling rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def gemm_flops(N, D, C):
    return 3 * 2.0 * N * D * C


def quant_bytes(rows, cols, src_bytes, fused=True):
    # source read + codes and scales of each output layout
    return rows * cols * (src_bytes + (2 if fused else 1) * (0.5 + 1.0 / 32))


def cpu_baseline(layers, sample_tokens):
    """The oracle, as it stands, on the first `sample_tokens` tokens of every layer."""
    import numpy as np
    import mx_workloads as wl
    from oracle import mx_oracle as orc
    orc.lib()
    flops = 0.0
    data = []
    for (name, N, D, C) in layers:
        X, W, dY = wl.linear_layer(sample_tokens, D, C, seed=0, dtype="bf16")
        data.append((X, W, dY))
        flops += gemm_flops(sample_tokens, D, C)
    t0 = time.perf_counter()
    for (X, W, dY) in data:
        xt = orc.quantize_transposed(X, round_t=1, tensor_id_t=6, pre_quant=1, round_row=0, tensor_id_row=1, seed=0)
        wt = orc.quantize_transposed(W, round_t=1, tensor_id_t=4, pre_quant=1, round_row=0, tensor_id_row=2, seed=0)
        dy = orc.quantize_transposed(dY, round_t=1, tensor_id_t=5, pre_quant=0, round_row=1, tensor_id_row=3, seed=0)
        orc.gemm_f64(xt[2], xt[3], wt[2], wt[3])
        orc.gemm_f64(dy[2], dy[3], wt[0], wt[1])
        orc.gemm_f64(dy[0], dy[1], xt[0], xt[1])
    dt = time.perf_counter() - t0
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": "first %d tokens of each of the %d layers (quantizers + FP64 products), %.1f s" % (
                sample_tokens, len(layers), dt)}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    import mx_workloads as wl
    import paper_2502_20853_amd as mx
    mx.binding.lib()                       # fails loudly if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    layers = wl.config_layers(args.workload, args.tokens)
    cfg = wl.CONFIGS[args.workload]
    steps_obj, inputs = [], []
    for li, (name, N, D, C) in enumerate(layers):
        X, W, dY = wl.device_linear_layer(N, D, C, seed=li, dtype=cfg["dtype"], outliers=cfg["outliers"])
        inputs.append((X, W, dY))
        steps_obj.append(mx.MxLinearStep(N, D, C, out_dtype=torch.bfloat16, dw_dtype=torch.float32))
    torch.cuda.synchronize()

    total_flops = sum(gemm_flops(N, D, C) for (_, N, D, C) in layers)
    sb = 2 if cfg["dtype"] == "bf16" else 4
    q_bytes = sum(quant_bytes(N, D, sb) + quant_bytes(C, D, sb) + quant_bytes(N, C, sb) for (_, N, D, C) in layers)

    ev = lambda: torch.cuda.Event(enable_timing=True)
    gemm_events, quant_events = [], []
    per_launch = {}                        # (layer index, op) -> list of (start, end) events

    side_stream = torch.cuda.Stream()                                # default priority
    dw_ws = [torch.empty_like(st.workspace) for st in steps_obj]     # the dW product's own K-split workspace

    def run_step(seed, record, side=None):
        """One step.  With one stream (side is None) every launch follows the previous one, and per-kernel
        events may be recorded.  With two, MxLinearStep.step_two_streams spreads a layer's launches over
        the current stream and `side`, so that the tail of one kernel overlaps the next."""
        assert not (record and side is not None)
        B = mx.binding
        main = torch.cuda.current_stream()
        for li, (st, (X, W, dY)) in enumerate(zip(steps_obj, inputs)):
            e = [ev() for _ in range(12)] if record else None
            if side is None:
                if record: e[0].record()
                st.quantize_inputs(X, W, seed)         # Q1/Q6 of X and Q2/Q4 of W in one launch
                if record: e[2].record()
                B.mx_linear_fwd(st.xq, st.xs, st.wq, st.ws, out=st.y, workspace=st.workspace)
                if record: e[3].record()
                B.mx_quantize_transposed(dY, B.ROUND_SR, 5, 0, True, B.ROUND_SR, 3, seed=seed, out=(st.dytq, st.dyts, st.dyq, st.dys))
                if record: e[4].record()
                B.mx_linear_bwd_dx(st.dyq, st.dys, st.wtq, st.wts, out=st.dx, workspace=st.workspace)
                if record: e[5].record()
                B.mx_linear_bwd_dw(st.dytq, st.dyts, st.xtq, st.xts, out=st.dw, workspace=st.workspace)
                if record: e[6].record()
                spans = {"quant X+W": (0, 2), "fwd": (2, 3), "quant dY": (3, 4), "dX": (4, 5), "dW": (5, 6)}
            else:
                st.step_two_streams(X, W, dY, seed, side, dw_ws[li])      # no events: see layer.py for the schedule
            if record:
                quant_events.extend([(e[a], e[b]) for k, (a, b) in spans.items() if k.startswith("quant")])
                gemm_events.extend([(e[a], e[b]) for k, (a, b) in spans.items() if not k.startswith("quant")])
                for op, (a, b) in spans.items():
                    per_launch.setdefault((li, op), []).append((e[a], e[b]))

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB read, 1 GiB written
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        mx.binding.mx_calibration_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    timed_side = side_stream if args.streams == 2 else None
    board = BoardPower()
    board.start()                          # sampled through the settle phase, the warm-up and the timed steps
    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
        for w in range(5):
            run_step(w, False, None)
        torch.cuda.synchronize()
    for w in range(args.warmup):
        run_step(w, False, timed_side)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    n_recorded = 0
    for s in range(args.steps):
        rec = s % max(1, args.event_every) == 0
        n_recorded += rec
        # events are recorded on the stream each kernel is launched on; a step that carries them runs on one
        # stream, so that the interval between a kernel's two events holds no other kernel's work
        run_step(1000 + s, rec, None if rec else timed_side)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    step_watts = board.stop(since=t_settle + 0.1)

    # the same steps under the other schedule, after the timed region, for comparison: with two
    # streams the tails of the products overlap the next kernels, but a kernel's event-to-event time
    # then includes the time it shares the chip, so the per-kernel figures come from one stream
    other_ms = None
    if not args.no_other_schedule:
        other_side = None if args.streams == 2 else side_stream
        for w in range(2):
            run_step(w, False, other_side)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for s in range(args.steps):
            run_step(2000 + s, False, other_side)
        torch.cuda.synchronize()
        other_ms = (time.perf_counter() - t1) * 1e3 / args.steps

    # the same step recorded once into a HIP graph and replayed: the seed lives in device memory and
    # is advanced inside the graph, so every replay rounds with new numbers (one stream, no events)
    graph_ms = None
    if not args.no_other_schedule:
        try:
            seed_t = torch.full((1,), 3000, dtype=torch.int64, device="cuda")
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for st, (X, W, dY) in zip(steps_obj, inputs):
                    st.forward(X, W, seed_t)
                    st.backward(dY, seed_t)
                seed_t.add_(1)
            for w in range(2):
                graph.replay()
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            for s in range(args.steps):
                graph.replay()
            torch.cuda.synchronize()
            graph_ms = (time.perf_counter() - t2) * 1e3 / args.steps
            del graph
        except Exception as exc:                           # reported, never fatal to the measurement above
            graph_ms = "failed: %s" % (exc,)

    # forward product with the layer's bias added in its output stage, against the bare product and
    # against the bare product followed by a separate add (outside the timed region)
    fwd_bias = []
    B = mx.binding
    if not args.no_other_schedule:
        for (name, N, D, C), st in zip(layers, steps_obj):
            bias = torch.randn(C, device="cuda")
            bias_out = bias.to(st.y.dtype)
            runs = {"fused_us": lambda: B.mx_linear_fwd_bias(st.xq, st.xs, st.wq, st.ws, bias, out=st.y, workspace=st.workspace),
                    "bare_us": lambda: B.mx_linear_fwd(st.xq, st.xs, st.wq, st.ws, out=st.y, workspace=st.workspace),
                    "bare_then_add_us": lambda: B.mx_linear_fwd(st.xq, st.xs, st.wq, st.ws, out=st.y, workspace=st.workspace).add_(bias_out)}
            row = {"layer": name, "shape": [N, C, D]}
            for key, fn in runs.items():
                for _ in range(3):
                    fn()
                e0, e1 = ev(), ev()
                e0.record()
                for _ in range(10):
                    fn()
                e1.record()
                torch.cuda.synchronize()
                row[key] = round(e0.elapsed_time(e1) / 10 * 1e3, 1)
            fwd_bias.append(row)

    # What the matrix cores sustain on given operand bytes, outside the timed region: the products' MFMA in
    # a register-resident loop (no LDS, no memory), one workgroup of 8 waves per compute unit, about a
    # millisecond per launch, on constant bytes, on uniformly random bytes and on the packed codes of this
    # workload's activations.  A calibration figure next to the roofline, never its peak.
    mfma_cal = {}
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    gen_cal = torch.Generator(device="cuda").manual_seed(11)
    need = mx.binding.CALIBRATION_MFMA_OPERAND_BYTES
    cal_inputs = {"constant_bytes_0x22": torch.full((need,), 0x22, dtype=torch.uint8, device="cuda"),
                  "random_bytes": torch.randint(0, 256, (need,), dtype=torch.uint8, device="cuda", generator=gen_cal),
                  "quantized_activation_codes": steps_obj[0].xq.reshape(-1)[:need].contiguous()}
    cal_sink = torch.empty(n_cu * 512, dtype=torch.float32, device="cuda")
    for key, ops in cal_inputs.items():
        for _ in range(2):
            mx.binding.mx_calibration_mfma(ops, n_cu, 2000, cal_sink)
        e0, e1 = ev(), ev()
        e0.record()
        fl = 0.0
        for _ in range(3):
            fl += mx.binding.mx_calibration_mfma(ops, n_cu, 2000, cal_sink)
        e1.record()
        torch.cuda.synchronize()
        mfma_cal[key] = round(fl / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
    # Board power (amdgpu hwmon) while one kernel family runs back to back for 0.4 s each, against the board's
    # power cap: the products, the quantizers and the calibration loop each draw close to the cap on their
    # own, which is what sets the shader clock they run at.
    def products_only():
        B = mx.binding
        for st in steps_obj:
            B.mx_linear_fwd(st.xq, st.xs, st.wq, st.ws, out=st.y, workspace=st.workspace)
            B.mx_linear_bwd_dx(st.dyq, st.dys, st.wtq, st.wts, out=st.dx, workspace=st.workspace)
            B.mx_linear_bwd_dw(st.dytq, st.dyts, st.xtq, st.xts, out=st.dw, workspace=st.workspace)

    def quantizers_only():
        B = mx.binding
        for st, (X, W, dY) in zip(steps_obj, inputs):
            st.quantize_inputs(X, W, 7)
            B.mx_quantize_transposed(dY, B.ROUND_SR, 5, 0, True, B.ROUND_SR, 3, seed=7, out=(st.dytq, st.dyts, st.dyq, st.dys))

    sync = torch.cuda.synchronize
    if args.no_power:
        board.path = None
    power = {"unit": "W", "source": "amdgpu hwmon power1_input, 10 ms samples", "cap": board.cap_w,
             "whole_step": step_watts,
             "products_only": board.watts_of(products_only, sync),
             "quantizers_only": board.watts_of(quantizers_only, sync),
             "calibration_mfma_constant_bytes": board.watts_of(
                 lambda: mx.binding.mx_calibration_mfma(cal_inputs["constant_bytes_0x22"], n_cu, 2000, cal_sink), sync),
             "calibration_mfma_quantized_codes": board.watts_of(
                 lambda: mx.binding.mx_calibration_mfma(cal_inputs["quantized_activation_codes"], n_cu, 2000, cal_sink), sync)}
    mfma_cal.update({"unit": "TFLOP/s", "kernel": "calibration_mfma_kernel", "workgroups": n_cu, "waves_per_simd": 2,
                     "note": "register-resident V_MFMA_SCALE_F32_32X32X64_F8F6F4 loop; calibration only, not the roofline peak"})

    # fc1 -> GELU -> fc2's quantizers, outside the timed region: the fused forward product (GELU and fc2's Q1
    # in fc1's output stage, fc2's Q6 from the packed codes) against the separate calls (forward product with
    # bias, an element-wise GELU kernel, the fused Q1/Q6 quantizer reading the activation)
    mlp_fusion = None
    # (the fused stage lives in the main product kernel: K a multiple of 128, at least 512, output width % 32)
    fusable = (len(layers) >= 4 and [n for (n, _, _, _) in layers[2:4]] == ["fc1", "fc2"]
               and layers[2][2] % 128 == 0 and layers[2][2] >= 512 and layers[2][3] % 32 == 0)
    if not args.no_other_schedule and fusable:
        (_, N1, D1, C1), st1, st2 = layers[2], steps_obj[2], steps_obj[3]
        bias1 = torch.randn(C1, device="cuda") * 0.1
        gelu = torch.nn.functional.gelu
        act = gelu(st1.y)

        def sep_product():
            B.mx_linear_fwd_bias(st1.xq, st1.xs, st1.wq, st1.ws, bias1, out=st1.y, workspace=st1.workspace)

        def sep_quant():
            B.mx_quantize_transposed(act, B.ROUND_SR, 6, 1, True, B.ROUND_RTN, 1, seed=1, out=(st2.xtq, st2.xts, st2.xq, st2.xs))

        def separate():
            sep_product()
            a = gelu(st1.y)                                # (torch's allocator hands back the same block each time)
            B.mx_quantize_transposed(a, B.ROUND_SR, 6, 1, True, B.ROUND_RTN, 1, seed=1, out=(st2.xtq, st2.xts, st2.xq, st2.xs))

        def fused_product():
            B.mx_linear_fwd_gelu_quant(st1.xq, st1.xs, st1.wq, st1.ws, bias1, out=st1.y, quant_out=(st2.xq, st2.xs))

        def q6_from_codes():
            B.mx_quantize_transposed(None, B.ROUND_SR, 6, 1, False, row_in=(st2.xq, st2.xs), seed=1, shape=(N1, C1),
                                     out=(st2.xtq, st2.xts, None, None))

        def fused():
            fused_product()
            q6_from_codes()

        mlp_fusion = {"layer": "fc1 -> GELU -> fc2 quantizers", "shape": [N1, C1, D1]}
        for key, fn in (("separate_us", separate), ("fused_us", fused), ("separate_product_us", sep_product),
                        ("separate_gelu_us", lambda: gelu(st1.y)), ("separate_quantizer_us", sep_quant),
                        ("fused_product_us", fused_product), ("fused_q6_from_codes_us", q6_from_codes)):
            for _ in range(3):
                fn()
            e0, e1 = ev(), ev()
            e0.record()
            for _ in range(10):
                fn()
            e1.record()
            torch.cuda.synchronize()
            mlp_fusion[key] = round(e0.elapsed_time(e1) / 10 * 1e3, 1)
        del act

    # E3M0 element codec of the format ablation (Table 7), outside the timed region: the row quantizer on the
    # largest activation of the block, both rounding rules, next to the E2M1 row quantizer on the same tensor
    # (algorithmic bytes: source + 0.5 B codes + 1/32 B scales per element)
    e3m0 = []
    Xl = max((X for (X, _, _) in inputs), key=lambda t: t.numel())
    qb_row = Xl.numel() * (Xl.element_size() + 0.5 + 1.0 / 32)
    e3_out = (torch.empty((Xl.shape[0], Xl.shape[1] // 2), dtype=torch.uint8, device="cuda"),
              torch.empty((Xl.shape[0], Xl.shape[1] // 32), dtype=torch.uint8, device="cuda"))
    for label, fn in (("e3m0 round_D", lambda: mx.binding.mx_quantize_e3m0(Xl, mx.binding.ROUND_RTN, out=e3_out)),
                      ("e3m0 round_S", lambda: mx.binding.mx_quantize_e3m0(Xl, mx.binding.ROUND_SR, seed=9, tensor_id=6, out=e3_out)),
                      ("e2m1 round_D", lambda: mx.binding.mx_quantize(Xl, mx.binding.ROUND_RTN, out=e3_out)),
                      ("e2m1 round_S", lambda: mx.binding.mx_quantize(Xl, mx.binding.ROUND_SR, seed=9, tensor_id=6, out=e3_out))):
        for _ in range(2):
            fn()
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(10):
            fn()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / 10 * 1e3
        e3m0.append({"op": label, "shape": list(Xl.shape), "us": round(us, 1), "GB/s": round(qb_row / us / 1e3, 1),
                     "hbm_frac": round(qb_row / us / 1e3 / PEAK_HBM_GBS, 3)})
    del e3_out

    # Q-EMA weight quantizer (Sec. 5), outside the timed region: the four weights of the block, one
    # update + quantization each, as a training step with Q-EMA would issue them
    qema = []
    for (name, N, D, C), (X, W, dY) in zip(layers, inputs):
        w32 = W.float()
        ema = w32.clone()
        out = (torch.empty((C, D // 2), dtype=torch.uint8, device="cuda"), torch.empty((C, D // 32), dtype=torch.uint8, device="cuda"))
        for _ in range(3):
            mx.binding.mx_ema_weight_quant(w32, ema, 0.998, 1, out=out)
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(20):
            mx.binding.mx_ema_weight_quant(w32, ema, 0.998, 1, out=out)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / 20 * 1e3
        qema.append({"layer": name, "shape": [C, D], "us": round(us, 1),
                     "GB/s": round(C * D * (4 + 4 + 4 + 0.5 + 1.0 / 32) / us / 1e3, 1)})

    # Q-Ramping's oscillation detection (Sec. 6.1) and amplification factor (Algorithm 2), also
    # outside the timed region: one accumulation step and one factor pass per weight of the block
    osc = []
    for (name, N, D, C), (X, W, dY) in zip(layers, inputs):
        w32 = W.float()
        codes, scales = mx.binding.mx_quantize(W)
        st = mx.binding.OscillationState(C, D)
        mx.binding.mx_oscillation_accumulate(w32, codes, scales, st, init=True)
        fac = mx.binding.mx_ramping_factor(st.dist_w, st.dist_q)
        for _ in range(3):
            mx.binding.mx_oscillation_accumulate(w32, codes, scales, st, init=False)
        e0, e1, e2 = ev(), ev(), ev()
        e0.record()
        for _ in range(20):
            mx.binding.mx_oscillation_accumulate(w32, codes, scales, st, init=False)
        e1.record()
        for _ in range(20):
            mx.binding.mx_ramping_factor(st.dist_w, st.dist_q, out=fac)
        e2.record()
        torch.cuda.synchronize()
        us_a, us_f = e0.elapsed_time(e1) / 20 * 1e3, e1.elapsed_time(e2) / 20 * 1e3
        osc.append({"layer": name, "shape": [C, D], "accumulate_us": round(us_a, 1),
                    "accumulate_GB/s": round(C * D * (4 + 8 + 3 * (0.5 + 1.0 / 32) + 16) / us_a / 1e3, 1),
                    "factor_us": round(us_f, 1), "factor_GB/s": round(C * D * 12 / us_f / 1e3, 1)})

    # oscillation diagnostics of Sec. 4 (quantization confidence with its histogram; one term of
    # the rate of change), outside the timed region, on each weight of the block
    diag = []
    for (name, N, D, C), (X, W, dY) in zip(layers, inputs):
        hist = torch.zeros(100, dtype=torch.int64, device="cuda")
        rs = mx.binding.RateOfChangeState(C, D)
        mx.binding.mx_rate_of_change_step(W, rs)
        for _ in range(3):
            mx.binding.mx_quant_confidence(W, conf=False, hist=hist)
            mx.binding.mx_rate_of_change_step(W, rs)
        e0, e1, e2 = ev(), ev(), ev()
        e0.record()
        for _ in range(20):
            mx.binding.mx_quant_confidence(W, conf=False, hist=hist)
        e1.record()
        for _ in range(20):
            mx.binding.mx_rate_of_change_step(W, rs)
        e2.record()
        torch.cuda.synchronize()
        us_c, us_r = e0.elapsed_time(e1) / 20 * 1e3, e1.elapsed_time(e2) / 20 * 1e3
        eb = W.element_size()
        diag.append({"layer": name, "shape": [C, D], "confidence_hist_us": round(us_c, 1),
                     "confidence_hist_GB/s": round(C * D * eb / us_c / 1e3, 1),
                     "rate_of_change_us": round(us_r, 1),
                     "rate_of_change_GB/s": round(C * D * (eb + 8) / us_r / 1e3, 1)})

    # Q-Ramping's customised AdamW (Algorithm 2), outside the timed region: one optimizer step over
    # all quantized-layer weights of a 12-block model of these shapes (one flat launch), with factors
    # from a synthetic oscillating minority, and the same without factors (plain AdamW)
    n_par = 12 * sum(C * D for (_, _, D, C) in layers)
    gen = torch.Generator(device="cuda").manual_seed(5)
    w_all = torch.randn(n_par, device="cuda", generator=gen) * 0.02
    g_all = torch.randn(n_par, device="cuda", generator=gen) * 1e-3
    fac_all = torch.where(torch.rand(n_par, device="cuda", generator=gen) < 0.02,
                          torch.full((n_par,), 6, dtype=torch.int32, device="cuda"),
                          torch.ones(n_par, dtype=torch.int32, device="cuda"))
    opt = []
    for label, fac, bytes_per in (("ramping", fac_all, 56), ("plain_adamw", None, 36)):
        ost = mx.binding.RampingAdamwState((n_par,), ramping=fac is not None)
        for _ in range(2):
            mx.binding.mx_ramping_adamw_step(w_all, g_all, ost, fac)
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(10):
            mx.binding.mx_ramping_adamw_step(w_all, g_all, ost, fac)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / 10 * 1e3
        opt.append({"mode": label, "elements": n_par, "us": round(us, 1), "bytes_per_element": bytes_per,
                    "GB/s": round(n_par * bytes_per / us / 1e3, 1),
                    "hbm_frac": round(n_par * bytes_per / us / 1e3 / PEAK_HBM_GBS, 3)})
    del w_all, g_all, fac_all, ost

    gemm_ms = sum(a.elapsed_time(b) for a, b in gemm_events) / n_recorded      # per step, all 12 products
    quant_ms = sum(a.elapsed_time(b) for a, b in quant_events) / n_recorded
    n_gemm = 3 * len(layers)
    achieved = total_flops / (gemm_ms * 1e-3) / 1e12
    # the same kernel without launch gaps and neighbours' tails: its average duration in a rocprofv3
    # kernel trace of this command (profiles/gemm_kernel_only.json), the figure the committed summary shows
    kernel_only = None
    kj = os.path.join(ROOT, "profiles", "gemm_kernel_only.json")
    if os.path.exists(kj) and args.workload == "vit_base_b256" and args.tokens is None:
        try:
            ko = json.load(open(kj))
            ko_tf = total_flops / n_gemm / (ko["avg_launch_us"] * 1e-6) / 1e12
            kernel_only = {"avg_launch_us": ko["avg_launch_us"], "achieved": ko_tf, "frac": ko_tf / PEAK_FP4_TFLOPS,
                           "source": "profiles/gemm_kernel_only.json (rocprofv3 --kernel-trace of this command)"}
        except Exception:
            kernel_only = None
    traffic = None
    if os.path.exists(args.traffic_json):
        try:
            tj = json.load(open(args.traffic_json))
            if tj.get("workload") == args.workload and args.tokens is None:
                traffic = tj.get("hbm_bytes_per_launch")
        except Exception:
            traffic = None

    # per launch: products in TFLOP/s against min(FP4 peak, algorithmic intensity x HBM peak) of the
    # shape; quantizers in GB/s of algorithmic bytes
    launches = []
    for (li, op), evs in per_launch.items():
        name, N, D, C = layers[li]
        us = sum(a.elapsed_time(b) for a, b in evs) / len(evs) * 1e3
        if op.startswith("quant"):
            shapes = {"quant X": [(N, D)], "quant W": [(C, D)], "quant X+W": [(N, D), (C, D)], "quant dY": [(N, C)]}[op]
            qb = sum(quant_bytes(r, c, sb) for r, c in shapes)
            launches.append({"layer": name, "op": op, "shape": [list(x) for x in shapes] if len(shapes) > 1 else list(shapes[0]),
                             "us": round(us, 1), "GB/s": round(qb / us / 1e3, 1)})
        else:
            m, n, k, ob = {"fwd": (N, C, D, 2), "dX": (N, D, C, 2), "dW": (C, D, N, 4)}[op]
            fl = 2.0 * m * n * k
            by = (m + n) * k * 17 / 32 + m * n * ob
            roof = min(PEAK_FP4_TFLOPS, fl / by * PEAK_HBM_GBS / 1e3)
            launches.append({"layer": name, "op": op, "shape": [m, n, k], "us": round(us, 1),
                             "TFLOP/s": round(fl / us / 1e6, 1), "shape_roofline_TFLOP/s": round(roof, 1)})

    # The quantizers are bound by the vector ALUs: VALU lane-operations per element counted by rocprofv3
    # (SQ_INSTS_VALU x 64 / elements, profiles/quantizer_valu.json) x elements per step / quantizer time,
    # against the plain VALU rate 256 CUs x 4 SIMDs x 16 lanes/clk x 2.4 GHz.
    quant_alu = None
    vj = os.path.join(ROOT, "profiles", "quantizer_valu.json")
    if os.path.exists(vj) and args.workload == "vit_base_b256" and args.tokens is None:
        try:
            per = json.load(open(vj))["valu_lane_ops_per_element"]
            ops = sum(per["x_type"] * (N * D + C * D) + per["dy_type"] * N * C for (_, N, D, C) in layers)
            peak = 256 * 4 * 16 * 2.4e9
            quant_alu = {"bound": "alu", "achieved": ops / (quant_ms * 1e-3) / 1e12, "peak": peak / 1e12,
                         "unit": "T lane-ops/s", "frac": ops / (quant_ms * 1e-3) / peak,
                         "lane_ops_per_element": per}
        except Exception:
            quant_alu = None

    out = {
        "metric": "MXFP4 linear fwd+bwd TFLOP/s at ViT-B shapes",
        "value": total_flops / (dt / args.steps) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "mxfp4",
        "data": "synthetic",
        "config": {"workload": "%s: N=%d tokens, layers %s, Y/dX bf16, dW f32" % (
            args.workload, layers[0][1], ",".join("%s %d->%d" % (n, d, c) for (n, _, d, c) in layers)),
            "quantizers": "Q1,Q2 RTN; Q3..Q6 stochastic (Philox4x32-10); truncation-free scale; double quantization",
            "arithmetic": "E2M1 elements x E8M0 group scales in the products, FP32 accumulation; %s sources" % cfg["dtype"],
            "streams": args.streams, "steps_with_kernel_events": n_recorded,
            "settle_ms_before_warmup": args.settle_ms,
            "schedule": ("steps without kernel events: two streams (quant W, quant dY, dW beside quant X, fwd, dX); "
                         "steps with kernel events: one stream") if args.streams == 2 else "one stream"},
        "roofline": {"bound": "mfma", "kernel": "mx_gemm_pingpong_kernel<false> (12 launches per step)",
                     "achieved": achieved, "peak": PEAK_FP4_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_FP4_TFLOPS,
                     "timing": "HIP events around each product on its stream, live in this run: event to event, "
                               "i.e. with the launch gap and, for a K-split product, its reduction kernel",
                     "flops_per_launch": total_flops / n_gemm, "avg_launch_ms": gemm_ms / n_gemm,
                     "kernel_only": kernel_only,
                     "traffic": traffic},
        "power": power,
        "quantizers": {"bound": "hbm", "achieved": q_bytes / (quant_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                       "unit": "GB/s", "frac": q_bytes / (quant_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                       "ms_per_step": quant_ms, "bytes_per_step": q_bytes, "alu": quant_alu},
        "gemm_ms_per_step": gemm_ms,
        "mfma_sustained": mfma_cal,
        "launches": launches,
        "forward_with_bias": fwd_bias,
        "mlp_fusion": mlp_fusion,
        "e3m0_codec": e3m0,
        "qema_weight_quant": qema,
        "oscillation_detection": osc,
        "other_schedule": None if other_ms is None else {
            "streams": 3 - args.streams, "ms_per_step": other_ms,
            "value": total_flops / (other_ms * 1e-3) / 1e12, "unit": "TFLOP/s"},
        "graph_replay": None if graph_ms is None else (
            {"error": graph_ms} if isinstance(graph_ms, str) else
            {"ms_per_step": graph_ms, "value": total_flops / (graph_ms * 1e-3) / 1e12, "unit": "TFLOP/s"}),
        "oscillation_diagnostics": diag,
        "ramping_adamw": opt,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(layers, args.cpu_sample_tokens)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
