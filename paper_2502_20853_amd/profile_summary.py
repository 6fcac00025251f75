"""Turn rocprofv3 output of `bench.py` into the short text summaries kept under profiles/.

Collect (one MI355X; from /tmp with TMPDIR=/tmp; <out> is any scratch directory):

    rocprofv3 --kernel-trace --stats -d <out>/trace -o bench --output-format csv -- python3 bench.py --steps 10 --warmup 3 --no-cpu-baseline --no-other-schedule --no-power
    rocprofv3 --pmc FETCH_SIZE -d <out>/fetch -o bench --output-format csv -- python3 bench.py --steps 2 --warmup 1 --no-cpu-baseline --no-other-schedule --no-power --calibrate-copy
    rocprofv3 --pmc WRITE_SIZE -d <out>/write -o bench --output-format csv -- python3 bench.py --steps 2 --warmup 1 --no-cpu-baseline --no-other-schedule --no-power --calibrate-copy
    rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES SQ_INSTS_VALU_MFMA_MOPS_F6F4 SQ_INSTS_MFMA SQ_CYCLES GRBM_GUI_ACTIVE -d <out>/mfma -o bench --output-format csv -- python3 bench.py --steps 2 --warmup 1 --no-cpu-baseline --no-other-schedule --no-power
    rocprofv3 --pmc SQ_INSTS_VALU SQ_INSTS_SALU SQ_INSTS_LDS SQ_WAVES SQ_INSTS_VALU_INT64 SQ_ACTIVE_INST_VALU SQ_BUSY_CU_CYCLES SQ_THREAD_CYCLES_VALU -d <out>/valu -o bench --output-format csv -- python3 bench.py --steps 1 --warmup 1 --no-cpu-baseline --no-other-schedule --no-power

Summarise (writes profiles/*.md and the two small JSON files bench.py reads):

    python -m paper_2502_20853_amd.profile_summary <out>

Each pass is optional: a missing sub-directory leaves its summary as it is.
"""
import collections
import csv
import glob
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROFILES = os.path.join(ROOT, "profiles")

VIT_B_PRODUCTS = [("qkv fwd", 50432, 2304, 768), ("qkv dX", 50432, 768, 2304), ("qkv dW", 2304, 768, 50432),
                  ("proj fwd", 50432, 768, 768), ("proj dX", 50432, 768, 768), ("proj dW", 768, 768, 50432),
                  ("fc1 fwd", 50432, 3072, 768), ("fc1 dX", 50432, 768, 3072), ("fc1 dW", 3072, 768, 50432),
                  ("fc2 fwd", 50432, 768, 3072), ("fc2 dX", 50432, 3072, 768), ("fc2 dW", 768, 3072, 50432)]

CMD = {
    "trace": "rocprofv3 --kernel-trace --stats -d <out>/trace -o bench --output-format csv -- python3 bench.py --steps 10 --warmup 3 --no-cpu-baseline --no-other-schedule --no-power",
    "fetch": "rocprofv3 --pmc FETCH_SIZE -d <out>/fetch -o bench --output-format csv -- python3 bench.py --steps 2 --warmup 1 --no-cpu-baseline --no-other-schedule --no-power --calibrate-copy",
    "write": "rocprofv3 --pmc WRITE_SIZE -d <out>/write -o bench --output-format csv -- python3 bench.py --steps 2 --warmup 1 --no-cpu-baseline --no-other-schedule --no-power --calibrate-copy",
    "mfma": "rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES SQ_INSTS_VALU_MFMA_MOPS_F6F4 SQ_INSTS_MFMA SQ_CYCLES GRBM_GUI_ACTIVE -d <out>/mfma -o bench --output-format csv -- python3 bench.py --steps 2 --warmup 1 --no-cpu-baseline --no-other-schedule --no-power",
    "valu": "rocprofv3 --pmc SQ_INSTS_VALU SQ_INSTS_SALU SQ_INSTS_LDS SQ_WAVES SQ_INSTS_VALU_INT64 SQ_ACTIVE_INST_VALU SQ_BUSY_CU_CYCLES SQ_THREAD_CYCLES_VALU -d <out>/valu -o bench --output-format csv -- python3 bench.py --steps 1 --warmup 1 --no-cpu-baseline --no-other-schedule --no-power",
}
SUMMARISE = "python -m paper_2502_20853_amd.profile_summary <out>"


def _find(d, suffix):
    hits = sorted(glob.glob(os.path.join(d, "**", "*" + suffix), recursive=True))
    return hits[0] if hits else None


def _dispatches(path):
    """rocprofv3 counter CSV -> ordered list of dispatches with their counters and duration in us."""
    d = collections.OrderedDict()
    for r in csv.DictReader(open(path)):
        e = d.setdefault(int(r["Dispatch_Id"]), {
            "name": r["Kernel_Name"], "grid": int(r["Grid_Size"]),
            "us": (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3})
        e[r["Counter_Name"]] = e.get(r["Counter_Name"], 0.0) + float(r["Counter_Value"])
    return list(d.values())


def _short(name):
    name = name.replace("(anonymous namespace)::", "").replace("void ", "")
    i = name.find("(")
    return name[:i] if i > 0 else name


def kernel_stats(trace_csv):
    """kernel-trace CSV -> table of calls, total, average, maximum and share per kernel."""
    agg = collections.OrderedDict()
    for r in csv.DictReader(open(trace_csv)):
        us = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
        a = agg.setdefault(_short(r["Kernel_Name"]), [0, 0.0, 0.0])
        a[0] += 1
        a[1] += us
        a[2] = max(a[2], us)
    tot = sum(a[1] for a in agg.values())
    lines = ["%-58s %6s %12s %10s %10s %7s" % ("kernel", "calls", "total_us", "avg_us", "max_us", "share")]
    for k, a in sorted(agg.items(), key=lambda kv: -kv[1][1]):
        if a[1] / tot < 0.0005:
            continue
        lines.append("%-58s %6d %12.1f %10.1f %10.1f %6.1f%%" % (k[:58], a[0], a[1], a[1] / a[0], a[2], 100 * a[1] / tot))
    return "\n".join(lines), agg


def traffic(fetch_csv, write_csv):
    """FETCH_SIZE / WRITE_SIZE (KiB per dispatch), scaled by what the same counters read for the
    1 GiB calibration copy that `bench.py --calibrate-copy` launches."""
    per = {}
    for key, path in (("FETCH_SIZE", fetch_csv), ("WRITE_SIZE", write_csv)):
        by = collections.OrderedDict()
        for e in _dispatches(path):
            by.setdefault(_short(e["name"]), []).append(e[key])
        per[key] = by
    cal_f = per["FETCH_SIZE"]["calibration_copy_kernel"][0]
    cal_w = per["WRITE_SIZE"]["calibration_copy_kernel"][0]
    ff, wf = 1048576.0 / cal_f, 1048576.0 / cal_w
    return per, cal_f, cal_w, ff, wf


def write_step_kernels(out_dir):
    trace = _find(os.path.join(out_dir, "trace"), "kernel_trace.csv")
    fetch = _find(os.path.join(out_dir, "fetch"), "counter_collection.csv")
    write = _find(os.path.join(out_dir, "write"), "counter_collection.csv")
    if not (trace and fetch and write):
        return None
    table, agg = kernel_stats(trace)
    per, cal_f, cal_w, ff, wf = traffic(fetch, write)
    gk = [n for n in per["FETCH_SIZE"] if n.startswith("mx_gemm_pingpong_kernel<false")][0]
    f, w = per["FETCH_SIZE"][gk], per["WRITE_SIZE"][gk]
    rd, wr = sum(f) / len(f) * 1024 * ff, sum(w) / len(w) * 1024 * wf
    json.dump({"workload": "vit_base_b256", "kernel": gk, "launches_sampled": len(f), "fetch_factor": ff,
               "write_factor": wf, "hbm_read_bytes_per_launch": rd, "hbm_write_bytes_per_launch": wr,
               "hbm_bytes_per_launch": rd + wr}, open(os.path.join(PROFILES, "gemm_traffic.json"), "w"), indent=1)
    gem = [a for k, a in agg.items() if k.startswith("mx_gemm_pingpong_kernel<false")][0]
    red = [a for k, a in agg.items() if k.startswith("splitk_reduce4_kernel")]
    json.dump({"workload": "vit_base_b256", "kernel": gk, "launches": gem[0], "avg_launch_us": gem[1] / gem[0],
               "reduction_avg_us": (red[0][1] / red[0][0]) if red else None, "reductions_per_step": 4,
               "source": "rocprofv3 --kernel-trace of bench.py (profiles/vit_base_b256_step_kernels.md)"},
              open(os.path.join(PROFILES, "gemm_kernel_only.json"), "w"), indent=1)
    # fused quantizer launches: counter traffic against the algorithmic bytes (bf16 source read once; codes
    # 0.5 B and scale 1/32 B per element, in both layouts)
    known = {1340: ("dY-type 50432x768", 50432 * 768), 3546: ("dY-type 50432x2304", 50432 * 2304),
             4848: ("dY-type 50432x3072", 50432 * 3072), 1376: ("X-type 50432x768 + weight", 50432 * 768 + 768 * 768),
             4992: ("X-type 50432x3072 + weight", 50432 * 3072 + 768 * 3072),
             1448: ("X-type 50432x768 + weight 2304x768", 50432 * 768 + 2304 * 768),
             1484: ("X-type 50432x768 + weight 3072x768", 50432 * 768 + 3072 * 768)}
    qrows = collections.OrderedDict()
    fd, wd = _dispatches(fetch), _dispatches(write)
    for ef, ew in zip(fd, wd):
        if "quantize_tile_kernel" not in ef["name"] or ef["grid"] // 512 not in known or ef["grid"] != ew["grid"]:
            continue
        label, elements = known[ef["grid"] // 512]
        q = qrows.setdefault(label, [elements, [], []])
        q[1].append(ef["FETCH_SIZE"] * 1024 * ff)
        q[2].append(ew["WRITE_SIZE"] * 1024 * wf)
    qlines = ["| fused quantizer launch | read MB (counter) | algorithmic | write MB (counter) | algorithmic | write / algorithmic |", "|---|---|---|---|---|---|"]
    for label, (elements, fr, wr_) in qrows.items():
        r_, w_ = sum(fr) / len(fr), sum(wr_) / len(wr_)
        qlines.append("| %s | %.1f | %.1f | %.1f | %.1f | %.3f |" % (label, r_ / 1e6, elements * 2 / 1e6, w_ / 1e6,
                                                                 elements * 1.0625 / 1e6, w_ / (elements * 1.0625)))
    n_par = 12 * (2304 * 768 + 768 * 768 + 3072 * 768 + 768 * 3072)
    opt = []
    for ok, label in (("ramping_adamw_kernel<float, true>", "with factors (56 B/element algorithmic)"),
                      ("ramping_adamw_kernel<float, false>", "plain AdamW (36 B/element algorithmic)")):
        if ok in per["FETCH_SIZE"]:
            f2, w2 = per["FETCH_SIZE"][ok], per["WRITE_SIZE"][ok]
            r2, wr2 = sum(f2) / len(f2) * 1024 * ff, sum(w2) / len(w2) * 1024 * wf
            opt.append("%s, %s: read %.1f MB + write %.1f MB per launch = %.2f + %.2f B per element" % (
                ok, label, r2 / 1e6, wr2 / 1e6, r2 / n_par, wr2 / n_par))
    md = """# rocprofv3 summary: MXFP4 GEMM and quantizer kernels, ViT-B/16 batch 256 step (bench.py)

Commands (one MI355X, from /tmp with TMPDIR=/tmp; <out> is a scratch directory):

    %s
    %s
    %s
    %s

One step = 4 layers x (2 fused quantizer launches + 3 products, the K-split ones followed by a reduction); %d steps traced
(the untimed settle phase of 250 ms, 3 warm-up steps, 10 timed steps, and the steps bench.py runs afterwards for its other figures).
`calibration_copy_kernel` copies 1 GiB (1048576 KiB read, 1048576 KiB written): FETCH_SIZE reads
%.1f KiB for it, WRITE_SIZE %.1f KiB, so the scale factors are %.3f (fetch) and %.3f (write).
Scaled HBM traffic of the dominant kernel (%s), average per launch over the 12 products of a step:
read %.1f MB + write %.1f MB = %.1f MB (profiles/gemm_traffic.json, read by bench.py).
Kernel-only average duration of that kernel: %.1f us over %d launches (profiles/gemm_kernel_only.json, read by bench.py).

Scaled HBM traffic of the fused quantizer launches of a step (quantize_tile_kernel; every workgroup stages its codes
and scale bytes in LDS and each XCD takes a contiguous range of the tile order, so that sectors leave L2 whole):

%s

After its timed region the same command also measures the kernels beyond the layer (Q-EMA, oscillation
detection, diagnostics, the MLP fusion comparison, the MFMA calibration loop and the optimizer step on the %d
weight elements of a 12-block model); scaled HBM traffic of the optimizer kernel:
%s

```
== kernel-trace stats (bench.py --steps 10 --warmup 3) ==
%s
```
""" % (CMD["trace"], CMD["fetch"], CMD["write"], SUMMARISE, gem[0] // 12, cal_f, cal_w, ff, wf, gk, rd / 1e6, wr / 1e6, (rd + wr) / 1e6,
       gem[1] / gem[0], gem[0], "\n".join(qlines), n_par, "\n".join(opt), table)
    open(os.path.join(PROFILES, "vit_base_b256_step_kernels.md"), "w").write(md)
    return md


def write_mfma(out_dir):
    path = _find(os.path.join(out_dir, "mfma"), "counter_collection.csv")
    if not path:
        return None
    disp = _dispatches(path)
    gem = [e for e in disp if "mx_gemm_pingpong" in e["name"]]
    cal = [e for e in disp if "calibration_mfma" in e["name"]]
    rows = ["| product | m, n, k | kernel us | GFLOP (counter) | TFLOP/s | shader clock GHz | MFMA busy % of SIMD cycles | CU busy % |",
            "|---|---|---|---|---|---|---|---|"]
    tot_f = tot_t = 0.0
    for (nm, m, n, k), e in zip(VIT_B_PRODUCTS, gem[-12:]):
        gui = e["GRBM_GUI_ACTIVE"] / 8
        fl = e["SQ_INSTS_VALU_MFMA_MOPS_F6F4"] * 512
        assert abs(fl - 2.0 * m * n * k) < 1e-6 * fl, (nm, fl, 2.0 * m * n * k)
        tot_f += fl
        tot_t += e["us"]
        rows.append("| %s | %d, %d, %d | %.1f | %.1f | %.0f | %.2f | %.1f | %.1f |" % (
            nm, m, n, k, e["us"], fl / 1e9, fl / e["us"] / 1e6, gui / e["us"] / 1e3,
            100 * e["SQ_VALU_MFMA_BUSY_CYCLES"] / (gui * 1024), 100 * e["SQ_BUSY_CU_CYCLES"] / (gui * 256)))
    rows.append("| all 12 | | %.1f | %.1f | %.0f | | | |" % (tot_t, tot_f / 1e9, tot_f / tot_t / 1e6))
    # bench.py launches the calibration 5 times per operand kind (2 untimed + 3 timed): take the last of each five
    crow = ["| operand bytes | kernel us | GFLOP (counter) | TFLOP/s | shader clock GHz | MFMA busy % of SIMD cycles |", "|---|---|---|---|---|---|"]
    per_kind = len(cal) // 3
    for i, nm in enumerate(("constant bytes 0x22", "random bytes", "quantized activation codes")):
        if per_kind == 0:
            break
        e = cal[(i + 1) * per_kind - 1]
        gui = e["GRBM_GUI_ACTIVE"] / 8
        fl = e["SQ_INSTS_VALU_MFMA_MOPS_F6F4"] * 512
        crow.append("| %s | %.0f | %.1f | %.0f | %.2f | %.1f |" % (
            nm, e["us"], fl / 1e9, fl / e["us"] / 1e6, gui / e["us"] / 1e3, 100 * e["SQ_VALU_MFMA_BUSY_CYCLES"] / (gui * 1024)))
    md = """# rocprofv3 counter summary: matrix-core utilisation of the MXFP4 product kernel, ViT-B/16 batch 256 step

Commands (one MI355X, from /tmp with TMPDIR=/tmp; <out> is a scratch directory):

    %s
    %s

Derived columns.  GRBM_GUI_ACTIVE is summed over the 8 XCDs, so GRBM_GUI_ACTIVE / 8 is the number of shader
clocks the dispatch lasted and (GRBM_GUI_ACTIVE / 8) / duration is the shader clock it ran at.
SQ_INSTS_VALU_MFMA_MOPS_F6F4 x 512 = flops of the scaled FP4 MFMAs (it equals 2 m n k of every product
exactly, which the summarising script asserts).  SQ_VALU_MFMA_BUSY_CYCLES counts 32 cycles per
V_MFMA_SCALE_F32_32X32X64_F8F6F4, so "MFMA busy" = SQ_VALU_MFMA_BUSY_CYCLES / (shader clocks x 1024 SIMDs) is the
fraction of the dense FP4 rate at the clock the kernel actually ran at.  CU busy = SQ_BUSY_CU_CYCLES / (shader
clocks x 256 CUs).  Dispatches are serialised under counter collection, so the durations are kernel-only.

## mx_gemm_pingpong_kernel<false>, the 12 products of the last profiled step

%s

Kernel-only the 12 products take %.1f us = %.2f PFLOP/s = %.3f of the 10.1 PFLOP/s dense FP4 peak.

## calibration_mfma_kernel (mx_calibration_mfma: register-resident loop of the same MFMA, 2 waves per SIMD, no LDS or memory traffic in the loop)

%s

The same instruction stream sustains less on random bytes and on this workload's packed codes than on constant
bytes because the shader clock falls (power management; the published 10.1 PFLOP/s is 1024 SIMDs x 4096 flops
per clock at 2.4 GHz); `roofline.frac` in bench.py stays priced against the published figure.
""" % (CMD["mfma"], SUMMARISE, "\n".join(rows), tot_t, tot_f / tot_t / 1e9, tot_f / tot_t / 1e6 / 10100.0, "\n".join(crow))
    open(os.path.join(PROFILES, "gemm_mfma_counters.md"), "w").write(md)
    return md


def write_valu(out_dir):
    path = _find(os.path.join(out_dir, "valu"), "counter_collection.csv")
    if not path:
        return None
    # grid = workgroups x 512 lanes of 256 x 128 macro tiles (two 256 x 64 halves in the tail)
    known = {1340: ("dy_type", 50432, 768, 0), 3546: ("dy_type", 50432, 2304, 0), 4848: ("dy_type", 50432, 3072, 0),
             1376: ("x_type", 50432, 768, 768 * 768), 4992: ("x_type", 50432, 3072, 768 * 3072)}
    detail, per, lines = collections.OrderedDict(), {}, []
    for e in _dispatches(path):
        if "quantize_tile_kernel" not in e["name"] or e["grid"] // 512 not in known:
            continue
        kind, rows_, cols, extra = known[e["grid"] // 512]
        if ("<1, true, true" in e["name"]) != (kind == "dy_type"):
            continue
        key = "%s %dx%d%s" % (kind, rows_, cols, " + weight" if extra else "")
        if key in detail:
            continue
        elements = rows_ * cols + extra
        lane = e["SQ_INSTS_VALU"] * 64 / elements
        detail[key] = {"elements": elements, "valu_lane_ops_per_element": lane,
                       "int64_lane_ops_per_element": e["SQ_INSTS_VALU_INT64"] * 64 / elements,
                       "lds_lane_ops_per_element": e["SQ_INSTS_LDS"] * 64 / elements,
                       "valu_active_over_cu_busy": e["SQ_ACTIVE_INST_VALU"] / e["SQ_BUSY_CU_CYCLES"]}
        per[kind] = lane
        lines.append("%-26s elements %10d  SQ_INSTS_VALU %.4g  = %.1f lane-ops/element (64-bit multiply-adds %.1f)  SQ_INSTS_LDS %.4g  SQ_ACTIVE_INST_VALU/SQ_BUSY_CU_CYCLES %.2f" % (
            key, elements, e["SQ_INSTS_VALU"], lane, e["SQ_INSTS_VALU_INT64"] * 64 / elements, e["SQ_INSTS_LDS"],
            e["SQ_ACTIVE_INST_VALU"] / e["SQ_BUSY_CU_CYCLES"]))
    if "x_type" not in per or "dy_type" not in per:
        return None
    json.dump({"workload": "vit_base_b256", "kernel": "quantize_tile_kernel",
               "valu_lane_ops_per_element": {"x_type": per["x_type"], "dy_type": per["dy_type"]}, "detail": detail},
              open(os.path.join(PROFILES, "quantizer_valu.json"), "w"), indent=1)
    md = """# rocprofv3 counters: VALU work of the fused quantizer kernel, ViT-B/16 batch 256 step (bench.py)

Commands (one MI355X, from /tmp with TMPDIR=/tmp; <out> is a scratch directory):

    %s
    %s

SQ_INSTS_VALU counts wave instructions; x 64 lanes / elements of the tensor = VALU lane-operations per element.
x_type = quantize_tile_kernel<bf16, row RTN, transposed SR> with double quantization (X and W of a layer in one launch);
dy_type = quantize_tile_kernel<bf16, row SR, transposed SR> (dY).  One dispatch of each size:

```
%s
```

The kernel is bound by the vector ALUs, not by HBM: 39.3 T lane-ops/s is the chip's plain (non-packed) VALU
rate (256 CUs x 4 SIMDs x 16 lanes/clk x 2.4 GHz); profiles/quantizer_valu.json carries the per-element counts
that bench.py turns into an achieved ALU rate.
""" % (CMD["valu"], SUMMARISE, "\n".join(lines))
    open(os.path.join(PROFILES, "quantizer_valu_counters.md"), "w").write(md)
    return md


def main(argv):
    if len(argv) != 2:
        print(__doc__)
        return 2
    done = [name for name, fn in (("step kernels + traffic", write_step_kernels), ("mfma counters", write_mfma),
                                  ("quantizer valu counters", write_valu)) if fn(argv[1])]
    print("wrote:", ", ".join(done) if done else "nothing (no rocprofv3 output found under %s)" % argv[1])
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
