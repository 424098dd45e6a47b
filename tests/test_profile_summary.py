"""The rocprofv3-CSV -> text summariser: runs on small hand-made CSVs (no GPU, no profiler)."""
import csv
import json
import os

from paper_2512_07782_amd import profile_summary as ps

K = {
    "copy": "__amd_rocclr_copyBuffer",
    "fwd": "void gfwa::fwd_bf16_kernel<128>(bool _Accum const*, int)",
    "dkv": "void gfwa::bwd_dkv8_bf16_kernel<128, true>(bool _Accum const*, int)",
    "dq": "void gfwa::bwd_dq_spill_bf16_kernel<128>(bool _Accum const*, int)",
}


def write_counters(d, rows):
    os.makedirs(os.path.join(d, "vm"), exist_ok=True)
    with open(os.path.join(d, "vm", "1_counter_collection.csv"), "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(["Kernel_Name", "Counter_Name", "Counter_Value"])
        w.writerows(rows)


def test_hbm_traffic_scales_by_the_copy(tmp_path):
    fe, wr = str(tmp_path / "fetch"), str(tmp_path / "write")
    # a counter that reads half of what the copy moved: every kernel's figure must be doubled
    write_counters(fe, [(K["copy"], "FETCH_SIZE", 524288.0), (K["fwd"], "FETCH_SIZE", 1000.0), (K["fwd"], "FETCH_SIZE", 3000.0)])
    write_counters(wr, [(K["copy"], "WRITE_SIZE", 1048576.0), (K["fwd"], "WRITE_SIZE", 500.0), (K["fwd"], "WRITE_SIZE", 500.0)])
    text = ps.hbm_traffic(fe, wr)
    line = [l for l in text.splitlines() if l.startswith("forward ")]
    assert len(line) == 1
    _, fetch, write = line[0].split()
    assert float(fetch) == 2000.0 * 2.0 * 1024 and float(write) == 500.0 * 1024


def test_kernel_trace_and_sq_counters(tmp_path):
    kt = tmp_path / "kt"
    os.makedirs(kt / "vm")
    with open(kt / "vm" / "1_kernel_stats.csv", "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(["Name", "Calls", "TotalDurationNs", "AverageNs", "Percentage", "MinNs", "MaxNs", "StdDev"])
        w.writerow([K["fwd"], 10, 3400000, 340000.0, 50.0, 330000, 350000, 1.0])
        w.writerow([K["dkv"], 10, 6800000, 680000.0, 40.0, 670000, 690000, 1.0])
        w.writerow([K["dq"], 10, 2600000, 260000.0, 10.0, 250000, 270000, 1.0])
    log = tmp_path / "kt.log"
    log.write_text("noise\n" + json.dumps({"steps": 5, "warmup": 1, "config": {"workload": "test"}, "kernels": {"forward": {"avg_ms": 0.341}}}) + "\n")
    text = ps.kernel_trace(str(kt), str(log))
    row = [l for l in text.splitlines() if l.startswith("fwd_bf16_kernel<128>")][0].split()
    assert row[-1] == "341.0" and "340.0" in row
    a, b = str(tmp_path / "sqA"), str(tmp_path / "sqB")
    ra, rb = [], []
    for k in ("fwd", "dkv", "dq"):
        ra += [(K[k], "SQ_WAVE_CYCLES", 1000.0), (K[k], "SQ_WAIT_ANY", 250.0), (K[k], "SQ_WAIT_INST_ANY", 100.0),
               (K[k], "SQ_WAIT_INST_LDS", 10.0), (K[k], "SQ_BUSY_CYCLES", 1.0), (K[k], "SQ_VALU_MFMA_BUSY_CYCLES", 1.0),
               (K[k], "SQ_ACTIVE_INST_VALU", 1.0), (K[k], "SQ_ACTIVE_INST_LDS", 1.0)]
        rb += [(K[k], "SQ_INSTS_MFMA", 25.0), (K[k], "SQ_INSTS_VALU", 125.0), (K[k], "SQ_INSTS_LDS", 50.0),
               (K[k], "SQ_INSTS_SALU", 75.0), (K[k], "SQ_INSTS_VMEM", 5.0), (K[k], "SQ_LDS_BANK_CONFLICT", 0.0),
               (K[k], "SQ_LDS_IDX_ACTIVE", 100.0), (K[k], "SQ_ACTIVE_INST_ANY", 1.0)]
    write_counters(a, ra)
    write_counters(b, rb)
    text = ps.sq_counters(a, b, str(kt))
    busy = [l for l in text.splitlines() if l.startswith("matrix pipe busy")][0].split()
    assert [float(x) for x in busy[-3:]] == [0.4, 0.4, 0.4]          # 16 * 25 / 1000
    valu = [l for l in text.splitlines() if l.strip().startswith("of which VALU")][0].split()
    assert [float(x) for x in valu[-3:]] == [4.0, 4.0, 4.0]          # (125 - 25) / 25
