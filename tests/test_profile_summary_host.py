"""Host-side check of the rocprofv3 summariser on small synthetic CSV files (no GPU, no profiler)."""
import csv
import json
import os

from paper_2502_20853_amd import profile_summary as ps


def _write_counter_csv(path, dispatches):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(["Dispatch_Id", "Kernel_Name", "Grid_Size", "Start_Timestamp", "End_Timestamp", "Counter_Name", "Counter_Value"])
        for i, (name, grid, us, counters) in enumerate(dispatches, 1):
            for k, v in counters.items():
                w.writerow([i, name, grid, 1000 * i * 10000, 1000 * i * 10000 + int(us * 1000), k, v])


def test_mfma_summary_from_counters(tmp_path, monkeypatch):
    monkeypatch.setattr(ps, "PROFILES", str(tmp_path))
    disp = []
    for (_, m, n, k) in ps.VIT_B_PRODUCTS:
        fl = 2.0 * m * n * k
        us = fl / 3.0e9                                  # 3 PFLOP/s
        clocks = us * 2100.0                             # 2.1 GHz
        disp.append(("void (anonymous namespace)::mx_gemm_pingpong_kernel<false, false>(GemmArgs)", 131072, us,
                     {"GRBM_GUI_ACTIVE": clocks * 8, "SQ_INSTS_VALU_MFMA_MOPS_F6F4": fl / 512,
                      "SQ_VALU_MFMA_BUSY_CYCLES": 0.33 * clocks * 1024, "SQ_BUSY_CU_CYCLES": 0.7 * clocks * 256}))
    for _ in range(3 * 5):
        disp.append(("(anonymous namespace)::calibration_mfma_kernel(v4i const*, int, float*)", 131072, 1000.0,
                     {"GRBM_GUI_ACTIVE": 1000.0 * 1700 * 8, "SQ_INSTS_VALU_MFMA_MOPS_F6F4": 8.59e12 / 512,
                      "SQ_VALU_MFMA_BUSY_CYCLES": 0.94 * 1000.0 * 1700 * 1024, "SQ_BUSY_CU_CYCLES": 1000.0 * 1700 * 256}))
    _write_counter_csv(str(tmp_path / "out" / "mfma" / "bench_counter_collection.csv"), disp)
    md = ps.write_mfma(str(tmp_path / "out"))
    assert md is not None and os.path.exists(tmp_path / "gemm_mfma_counters.md")
    assert "| fc2 dW | 768, 3072, 50432 |" in md
    assert "| all 12 |" in md and "0.297 of the 10.1 PFLOP/s" in md
    assert md.count("| 2.10 | 33.0 | 70.0 |") == 12                 # clock, MFMA busy, CU busy columns
    assert "| quantized activation codes | 1000 |" in md and "| 1.70 | 94.0 |" in md


def test_missing_passes_leave_summaries_alone(tmp_path, monkeypatch):
    monkeypatch.setattr(ps, "PROFILES", str(tmp_path))
    os.makedirs(tmp_path / "empty")
    assert ps.write_step_kernels(str(tmp_path / "empty")) is None
    assert ps.write_mfma(str(tmp_path / "empty")) is None
    assert ps.write_valu(str(tmp_path / "empty")) is None
    assert os.listdir(tmp_path) == ["empty"]


def test_valu_summary_counts_lane_operations(tmp_path, monkeypatch):
    monkeypatch.setattr(ps, "PROFILES", str(tmp_path))
    def q(name, groups, elements, per_element):
        return (name, groups * 512, 100.0, {"SQ_INSTS_VALU": per_element * elements / 64, "SQ_INSTS_VALU_INT64": 5.0 * elements / 64,
                                           "SQ_INSTS_LDS": 1.7 * elements / 64, "SQ_INSTS_SALU": 1.0, "SQ_WAVES": 1.0,
                                           "SQ_ACTIVE_INST_VALU": 0.9, "SQ_BUSY_CU_CYCLES": 1.0, "SQ_THREAD_CYCLES_VALU": 1.0})
    dy = "void (anonymous namespace)::quantize_tile_kernel<1, true, true, false, false>(TileBatch)"
    xt = "void (anonymous namespace)::quantize_tile_kernel<1, false, true, false, false>(TileBatch)"
    _write_counter_csv(str(tmp_path / "out" / "valu" / "bench_counter_collection.csv"),
                       [q(dy, 4848, 50432 * 3072, 33.0), q(xt, 4992, 50432 * 3072 + 768 * 3072, 32.0)])
    md = ps.write_valu(str(tmp_path / "out"))
    assert md is not None
    j = json.load(open(tmp_path / "quantizer_valu.json"))
    assert abs(j["valu_lane_ops_per_element"]["dy_type"] - 33.0) < 1e-9
    assert abs(j["valu_lane_ops_per_element"]["x_type"] - 32.0) < 1e-9
