"""Turn rocprofv3 CSV output of ``bench.py`` runs into the short text summaries kept under ``profiles/``.

The summaries of the training workload come from five profiler runs of the same committed command, each
started from the repository root on the GPU machine (``cd /tmp && export TMPDIR=/tmp`` first; rocprofv3 of
ROCm 7.2; counters are collected in runs of their own, without any trace option)::

    rocprofv3 --kernel-trace --stats --output-format csv -d OUT/kt -- python3 bench.py --no-cpu-baseline --power-pass-seconds 0
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d OUT/fetch -- \\
        python3 bench.py --steps 5 --warmup 1 --no-cpu-baseline --no-peak-probe --power-pass-seconds 0 --copy-calibration-mib 1024
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d OUT/write -- \\
        python3 bench.py --steps 5 --warmup 1 --no-cpu-baseline --no-peak-probe --power-pass-seconds 0 --copy-calibration-mib 1024
    rocprofv3 --pmc SQ_WAVE_CYCLES SQ_BUSY_CYCLES SQ_WAIT_INST_ANY SQ_WAIT_INST_LDS SQ_WAIT_ANY \\
        SQ_VALU_MFMA_BUSY_CYCLES SQ_ACTIVE_INST_VALU SQ_ACTIVE_INST_LDS --output-format csv -d OUT/sqA -- \\
        python3 bench.py --steps 3 --warmup 1 --no-cpu-baseline --no-peak-probe --power-pass-seconds 0
    rocprofv3 --pmc SQ_INSTS_VALU SQ_INSTS_MFMA SQ_INSTS_LDS SQ_INSTS_SALU SQ_LDS_BANK_CONFLICT \\
        SQ_LDS_IDX_ACTIVE SQ_ACTIVE_INST_ANY SQ_INSTS_VMEM --output-format csv -d OUT/sqB -- \\
        python3 bench.py --steps 3 --warmup 1 --no-cpu-baseline --no-peak-probe --power-pass-seconds 0

and then, with the standard output of the first run saved as OUT/kt.log::

    python3 -m paper_2512_07782_amd.profile_summary kernel-trace OUT/kt OUT/kt.log  > profiles/bench_long_bwd_kernel_trace.txt
    (other workloads: the same trace with bench.py's arguments as a fourth argument, e.g. "--workload train_bwd --no-cpu-baseline --power-pass-seconds 0")
    python3 -m paper_2512_07782_amd.profile_summary hbm-traffic OUT/fetch OUT/write > profiles/hbm_traffic_long_bwd.txt
    python3 -m paper_2512_07782_amd.profile_summary sq-counters OUT/sqA OUT/sqB OUT/kt > profiles/sq_counters_long_bwd.txt

Nothing here touches the GPU or the library: CSV in, text out.
"""
from __future__ import annotations

import collections
import csv
import glob
import json
import os
import re
import sys

# demangled kernel name (template arguments kept) -> the name bench.py and the library's profile use
LIB = {
    "segment_sum_kernel<false, 0>": "scan_segment_sum",
    "scan_rows_kernel<false, 0>": "gate_prefix_scan",
    "fwd_bf16_kernel<128>": "forward",
    "rowdot_bf16_kernel<128>": "bwd_rowdot",
    "bwd_dkv8_bf16_kernel<128, true>": "bwd_dkv",
    "bwd_dq_spill_bf16_kernel<128>": "bwd_dq",
    "segment_sum_kernel<true, 1>": "gate_grad_segment_sum",
    "scan_rows_kernel<true, 1>": "gate_grad_scan",
    # the other head dimension and the backward with its minimum workspace
    "fwd_bf16_kernel<64>": "forward",
    "rowdot_bf16_kernel<64>": "bwd_rowdot",
    "bwd_dkv_bf16_kernel<64>": "bwd_dkv",
    "bwd_dq_bf16_kernel<64>": "bwd_dq",
    "bwd_dkv8_bf16_kernel<128, false>": "bwd_dkv",
    "bwd_dq_bf16_kernel<128>": "bwd_dq",
    # fp32 storage
    "fwd_f32_mfma_kernel<128>": "forward", "fwd_f32_mfma_kernel<64>": "forward", "fwd_f32_kernel": "forward",
    "rowdot_f32_kernel": "bwd_rowdot",
    "bwd_dkv_f32_mfma_kernel<128>": "bwd_dkv", "bwd_dkv_f32_mfma_kernel<64>": "bwd_dkv", "bwd_dkv_f32_kernel": "bwd_dkv",
    "bwd_dq_f32_mfma_kernel<128>": "bwd_dq", "bwd_dq_f32_mfma_kernel<64>": "bwd_dq", "bwd_dq_f32_kernel": "bwd_dq",
}
# the long_bwd workload of bench.py
B, H, N, D, W = 1, 32, 16384, 128, 1024
CAL = "plain f32 copy (calibration)"


def short(name: str) -> str:
    m = re.search(r"gfwa::(\w+<[^>]*>)", name)
    if m:
        return m.group(1)
    m = re.search(r"gfwa::(\w+)", name)
    if m:
        return m.group(1)
    if "bfloat16_copy" in name:
        return "torch f32->bf16 conversion (input set-up)"
    if "FillFunctor" in name:
        return "torch fill (calibration source)"
    if "copyBuffer" in name or "direct_copy" in name:
        return CAL
    return name[:70]


def one(pattern: str) -> str:
    hits = glob.glob(pattern, recursive=True)
    if not hits:
        raise SystemExit(f"no file matches {pattern}")
    return max(hits, key=os.path.getmtime)  # a directory that was written to twice: the latest run


def bench_line(log: str) -> dict:
    lines = [l for l in open(log) if l.startswith("{")]
    if not lines:
        raise SystemExit(f"{log} holds no bench.py JSON line")
    return json.loads(lines[-1]), lines[-1].strip()


def kernel_trace(kt_dir: str, log: str, bench_args: str = "--no-cpu-baseline --power-pass-seconds 0") -> str:
    stats = one(os.path.join(kt_dir, "**", "*_kernel_stats.csv"))
    bj, raw = bench_line(log)
    out = [
        f"rocprofv3 kernel trace of bench.py, workload {bj['config']['workload']}",
        "(one step = gate prefix scan + forward + backward if the workload has one), one MI355X.",
        "",
        "command (from the repository root; rocprofv3 of ROCm 7.2):",
        f"  rocprofv3 --kernel-trace --stats --output-format csv -d OUT/kt -- python3 bench.py {bench_args}",
        f"      (bench.py, in this order: the calibration loops, {bj['warmup']} + {bj['steps']} steps with an event between the calls,",
        f"       {bj['warmup']} warm-up + {bj['steps']} timed steps)",
        "summary made by: python3 -m paper_2512_07782_amd.profile_summary kernel-trace OUT/kt OUT/kt.log",
        "",
        "kernel_stats.csv (all launches of the run: the warm-up steps and the first steps after the calibration loops,",
        "slower while the clocks settle, are in rocprofv3's average), next to the average bench.py measured with HIP",
        "events around the launches of its breakdown pass in the same run.",
        "scan_rows_kernel<reverse, input> / segment_sum_kernel<reverse, input>: input 0 = one tensor, 1 = difference of two",
        "tensors.  probe_* are the calibration loops (matrix cores with constant / pseudo-random operands / attention mix, copy).",
        "",
        f"{'kernel':36s} {'calls':>5s} {'avg us':>9s} {'min us':>9s} {'max us':>9s} {'% time':>7s} {'bench.py avg us':>16s}",
    ]
    for r in csv.DictReader(open(stats)):
        s = short(r["Name"])
        b = bj["kernels"].get(LIB.get(s, ""), {}).get("avg_ms")
        out.append(f"{s:36.36s} {r['Calls']:>5s} {float(r['AverageNs']) / 1e3:9.1f} {float(r['MinNs']) / 1e3:9.1f} "
                   f"{float(r['MaxNs']) / 1e3:9.1f} {float(r['Percentage']):7.2f} "
                   f"{('%16.1f' % (b * 1e3)) if b else ' ' * 16}")
    out += ["", "bench.py line of that run (under the profiler):", raw]
    return "\n".join(out) + "\n"


def counters(pmc_dir: str) -> tuple[dict, int]:
    path = one(os.path.join(pmc_dir, "**", "*_counter_collection.csv"))
    acc = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        acc[(short(r["Kernel_Name"]), r["Counter_Name"])].append(float(r["Counter_Value"]))
    n = max(len(v) for v in acc.values())
    return {k: sum(v) / len(v) for k, v in acc.items()}, n


def hbm_traffic(fetch_dir: str, write_dir: str) -> str:
    fe, nf = counters(fetch_dir)
    wr, _ = counters(write_dir)
    fe = {k[0]: v for k, v in fe.items()}
    wr = {k[0]: v for k, v in wr.items()}
    gib_kib = 1048576.0
    ff, wf = gib_kib / fe[CAL], gib_kib / wr[CAL]
    bhn = B * H * N
    nseg = (N + 4095) // 4096
    spill = B * H * (N // 32) * ((W + 30) // 32 + 1) * 2048  # dS blocks kept for the dQ pass
    algo = {
        "scan_segment_sum": (4 * bhn, 8 * B * H * nseg),
        "gate_prefix_scan": (4 * bhn, 4 * bhn),
        "forward": (3 * bhn * D * 2 + 4 * bhn, bhn * D * 2 + 4 * bhn),
        "bwd_rowdot": (2 * bhn * D * 2, 4 * bhn),
        "bwd_dkv": (4 * bhn * D * 2 + 12 * bhn, 2 * bhn * D * 2 + 4 * bhn + spill),
        "bwd_dq": (bhn * D * 2 + spill, bhn * D * 2 + 4 * bhn),
        "gate_grad_segment_sum": (8 * bhn, 8 * B * H * nseg),
        "gate_grad_scan": (8 * bhn, 4 * bhn),
    }
    o = [
        "# HBM traffic per launch of every kernel of bench.py, workload long_bwd (B=1 H=32 N=16384 d=128 w=1024",
        "# bf16), one MI355X, from two rocprofv3 counter runs (from the repository root, ROCm 7.2):",
        "#   rocprofv3 --pmc FETCH_SIZE --output-format csv -d OUT/fetch -- \\",
        "#       python3 bench.py --steps 5 --warmup 1 --no-cpu-baseline --no-peak-probe --power-pass-seconds 0 --copy-calibration-mib 1024",
        "#   rocprofv3 --pmc WRITE_SIZE --output-format csv -d OUT/write -- \\",
        "#       python3 bench.py --steps 5 --warmup 1 --no-cpu-baseline --no-peak-probe --power-pass-seconds 0 --copy-calibration-mib 1024",
        "# summary made by: python3 -m paper_2512_07782_amd.profile_summary hbm-traffic OUT/fetch OUT/write",
        "# The backward runs with the dS-block workspace (bench.py's default): the dK/dV kernel writes, and the dQ kernel",
        f"# reads, {spill / 1e6:.1f} MB of bf16 dS blocks per launch; both are counted in the algorithmic bytes below.",
        f"# Counters are KiB per dispatch, averaged over the dispatches of each kernel (up to {nf}).",
        f"# Calibration: the plain 1 GiB f32 copy (reads 1048576 KiB, writes 1048576 KiB) read FETCH_SIZE = {fe[CAL]:.1f},",
        f"# WRITE_SIZE = {wr[CAL]:.1f}  ->  scale factors fetch x{ff:.4f}, write x{wf:.4f}.",
        "# The compulsory traffic of the backward pass proper (Q, K, V, O, dO, c, L in; dQ, dK, dV, dalpha out, every",
        f"# tensor once) is {(5 * bhn * D * 2 + 8 * bhn + 3 * bhn * D * 2 + 4 * bhn) / 1e6:.1f} MB; the dS blocks add 2 x {spill / 1e6:.1f} MB to it by design.",
        "#",
        "# raw counters and scaled bytes against the algorithmic bytes of one launch:",
        f"# {'kernel':22s} {'FETCH KiB':>11s} {'WRITE KiB':>11s} {'fetch MB':>9s} {'write MB':>9s} {'algo rd MB':>10s} "
        f"{'algo wr MB':>10s} {'fetch/algo':>10s} {'write/algo':>10s}",
    ]
    rows, tot = [], [0.0, 0.0]
    for s, name in LIB.items():
        if s not in fe:
            continue
        fb, wb = fe[s] * ff * 1024, wr[s] * wf * 1024
        ar, aw = algo[name]
        o.append(f"# {name:22s} {fe[s]:11.1f} {wr[s]:11.1f} {fb / 1e6:9.1f} {wb / 1e6:9.1f} {ar / 1e6:10.1f} {aw / 1e6:10.1f} "
                 f"{fb / ar:10.2f} {wb / aw:10.2f}")
        rows.append(f"{name} {fb:.0f} {wb:.0f}")
        if name.startswith("bwd_") or name.startswith("gate_grad"):
            tot[0] += fb
            tot[1] += wb
    o += [f"# backward kernels together: {tot[0] / 1e6:.1f} MB fetched, {tot[1] / 1e6:.1f} MB written", "#",
          "# machine-readable part (bench.py reads it): <kernel> <fetch bytes per launch> <write bytes per launch>"]
    return "\n".join(o + rows) + "\n"


def sq_counters(a_dir: str, b_dir: str, kt_dir: str) -> str:
    tab = collections.defaultdict(dict)
    n = 0
    for d in (a_dir, b_dir):
        c, n = counters(d)
        for (k, name), v in c.items():
            tab[k][name] = v
    dur = {}
    for r in csv.DictReader(open(one(os.path.join(kt_dir, "**", "*_kernel_stats.csv")))):
        dur[short(r["Name"])] = float(r["AverageNs"]) * 1e-9
    cols = [("fwd_bf16_kernel<128>", "fwd"), ("bwd_dkv8_bf16_kernel<128, true>", "bwd_dkv8"),
            ("bwd_dq_spill_bf16_kernel<128>", "bwd_dq_spill")]
    names = ["SQ_INSTS_MFMA", "SQ_INSTS_VALU", "SQ_INSTS_LDS", "SQ_INSTS_SALU", "SQ_INSTS_VMEM", "SQ_VALU_MFMA_BUSY_CYCLES",
             "SQ_LDS_IDX_ACTIVE", "SQ_LDS_BANK_CONFLICT", "SQ_WAVE_CYCLES", "SQ_BUSY_CYCLES", "SQ_WAIT_ANY", "SQ_WAIT_INST_ANY",
             "SQ_WAIT_INST_LDS", "SQ_ACTIVE_INST_VALU", "SQ_ACTIVE_INST_LDS"]
    o = [
        "SQ counters of the three MFMA kernels, workload long_bwd (B=1 H=32 N=16384 d=128 w=1024 bf16), one MI355X,",
        "backward with the dS-block workspace (bench.py's default), from two rocprofv3 counter runs (from the repository",
        "root, ROCm 7.2):",
        "  rocprofv3 --pmc SQ_WAVE_CYCLES SQ_BUSY_CYCLES SQ_WAIT_INST_ANY SQ_WAIT_INST_LDS SQ_WAIT_ANY SQ_VALU_MFMA_BUSY_CYCLES \\",
        "      SQ_ACTIVE_INST_VALU SQ_ACTIVE_INST_LDS --output-format csv -d OUT/sqA -- \\",
        "      python3 bench.py --steps 3 --warmup 1 --no-cpu-baseline --no-peak-probe --power-pass-seconds 0",
        "  rocprofv3 --pmc SQ_INSTS_VALU SQ_INSTS_MFMA SQ_INSTS_LDS SQ_INSTS_SALU SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE \\",
        "      SQ_ACTIVE_INST_ANY SQ_INSTS_VMEM --output-format csv -d OUT/sqB -- \\",
        "      python3 bench.py --steps 3 --warmup 1 --no-cpu-baseline --no-peak-probe --power-pass-seconds 0",
        "summary made by: python3 -m paper_2512_07782_amd.profile_summary sq-counters OUT/sqA OUT/sqB OUT/kt",
        f"Counter values are sums over the chip (256 CUs, 1024 SIMDs), averaged over the dispatches of each kernel (up to {n}).",
        "SQ_WAVE_CYCLES counts in units of four clock cycles, summed over the resident waves; these kernels keep two waves",
        "on every SIMD (1024 SIMDs, 2048 waves) for all but the tail of a launch.  An MFMA (32x32x16 bf16) occupies the",
        "matrix pipe of its SIMD for 32 cycles, so 'matrix pipe busy' = 32 x SQ_INSTS_MFMA / (4 x SQ_WAVE_CYCLES / 2) is the",
        "share of a SIMD's cycles in which its matrix pipe works, whatever the clock was, and 'implied clock' =",
        "4 x SQ_WAVE_CYCLES / 2048 / duration is the core clock the kernel ran at (durations: kernel-trace averages of the",
        "same command; the part lowers its clock under load, see the probe_* rows of the kernel trace).",
        "",
        f"{'':38s}" + "".join(f"{c[1]:>14s}" for c in cols),
    ]
    for nm in names:
        if any(nm in tab[c[0]] for c in cols):
            o.append(f"{nm:38s}" + "".join(f"{tab[c[0]].get(nm, float('nan')):14.0f}" for c in cols))
    o.append("")

    def row(label, f):
        o.append(f"{label:38s}" + "".join(f"{f(tab[c[0]], dur.get(c[0], float('nan'))):14.3f}" for c in cols))

    row("duration, us (kernel trace)", lambda t, d: d * 1e6)
    row("matrix pipe busy (of SIMD cycles)", lambda t, d: 16.0 * t["SQ_INSTS_MFMA"] / t["SQ_WAVE_CYCLES"])
    row("implied clock, GHz", lambda t, d: 4.0 * t["SQ_WAVE_CYCLES"] / 2048.0 / d / 1e9)
    row("LDS address pipe busy (of CU cycles)", lambda t, d: t["SQ_LDS_IDX_ACTIVE"] / (4.0 * t["SQ_WAVE_CYCLES"] / 8.0))
    row("non-MFMA instructions per MFMA", lambda t, d: (t["SQ_INSTS_VALU"] - t["SQ_INSTS_MFMA"] + t["SQ_INSTS_LDS"] +
                                                        t["SQ_INSTS_SALU"] + t["SQ_INSTS_VMEM"]) / t["SQ_INSTS_MFMA"])
    row("  of which VALU (without MFMA)", lambda t, d: (t["SQ_INSTS_VALU"] - t["SQ_INSTS_MFMA"]) / t["SQ_INSTS_MFMA"])
    row("  of which LDS", lambda t, d: t["SQ_INSTS_LDS"] / t["SQ_INSTS_MFMA"])
    row("  of which SALU", lambda t, d: t["SQ_INSTS_SALU"] / t["SQ_INSTS_MFMA"])
    row("wave time in s_waitcnt (WAIT_ANY)", lambda t, d: t["SQ_WAIT_ANY"] / t["SQ_WAVE_CYCLES"])
    row("wave time waiting to issue", lambda t, d: t["SQ_WAIT_INST_ANY"] / t["SQ_WAVE_CYCLES"])
    row("wave time waiting for LDS issue", lambda t, d: t["SQ_WAIT_INST_LDS"] / t["SQ_WAVE_CYCLES"])
    row("LDS bank conflict / LDS active", lambda t, d: t["SQ_LDS_BANK_CONFLICT"] / max(t["SQ_LDS_IDX_ACTIVE"], 1.0))
    return "\n".join(o) + "\n"


def main(argv: list[str]) -> int:
    if len(argv) >= 4 and argv[1] == "kernel-trace":
        sys.stdout.write(kernel_trace(argv[2], argv[3], *argv[4:5]))
    elif len(argv) >= 4 and argv[1] == "hbm-traffic":
        sys.stdout.write(hbm_traffic(argv[2], argv[3]))
    elif len(argv) >= 5 and argv[1] == "sq-counters":
        sys.stdout.write(sq_counters(argv[2], argv[3], argv[4]))
    else:
        sys.stderr.write(__doc__)
        return 2
    return 0


if __name__ == "__main__":
    raise SystemExit(main(sys.argv))
