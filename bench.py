#!/usr/bin/env python3
"""Benchmark of the GatedFWA hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: gate prefix scan,
fused forward, and backward (row-dot, dK/dV, dQ, gate-gradient scan).  The default workload is the
one the target is stated on: B=1, H=32, N=16384, d=128, w=1024, bf16.  Prints ONE JSON line.

metric/value: effective TFLOP/s on in-window FLOPs of forward + backward, nominal count
(4 + 10) * B*H*N*w*d, inputs resident in HBM.  Forward-only and backward-only figures and their
fraction of the bf16 MFMA peak are reported in "detail".
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0    # MI355X dense bf16 MFMA, published
PEAK_F32_TFLOPS = 157.3      # MI355X fp32 MFMA (and fp32 vector), published
PEAK_HBM_GBS = 8000.0


class BoardPower:
    """Board power and shader clock of the GPU under test, read (never written) from the amdgpu driver's hwmon and
    pp_dpm_sclk files while a load runs.  None of it is needed for the timing; absent files just give no figures."""

    def __init__(self, torch, sysfs="/sys/class/drm"):
        import glob
        self.power = self.cap = self.sclk = None
        try:
            p = torch.cuda.get_device_properties(0)
            bus = f"{p.pci_domain_id:04x}:{p.pci_bus_id:02x}:{p.pci_device_id:02x}.0"
        except Exception:
            bus = ""
        cards = sorted(glob.glob(os.path.join(sysfs, "card[0-9]*", "device")))
        mine = [c for c in cards if bus and os.path.realpath(c).lower().endswith(bus)] or (cards if len(cards) == 1 else [])
        for c in mine[:1]:
            for hw in sorted(glob.glob(os.path.join(c, "hwmon", "hwmon*"))):
                for name in ("power1_input", "power1_average"):
                    if self.power is None and os.path.exists(os.path.join(hw, name)):
                        self.power = os.path.join(hw, name)
                if os.path.exists(os.path.join(hw, "power1_cap")):
                    self.cap = os.path.join(hw, "power1_cap")
            if os.path.exists(os.path.join(c, "pp_dpm_sclk")):
                self.sclk = os.path.join(c, "pp_dpm_sclk")

    @staticmethod
    def _read(path):
        try:
            with open(path) as f:
                return f.read()
        except OSError:
            return None

    def watts(self):
        v = self._read(self.power) if self.power else None
        return float(v) / 1e6 if v and v.strip().isdigit() else None

    def cap_watts(self):
        v = self._read(self.cap) if self.cap else None
        return float(v) / 1e6 if v and v.strip().isdigit() else None

    def sclk_mhz(self):
        for line in (self._read(self.sclk) or "").splitlines() if self.sclk else ():
            if line.rstrip().endswith("*"):
                digits = "".join(ch for ch in line.split(":")[-1] if ch.isdigit())
                return float(digits) if digits else None
        return None

    def during(self, torch, launch, seconds, settle=0.3):
        """Run `launch` back to back for `seconds`; mean/max of the samples taken after the first `settle` seconds."""
        import threading
        if self.power is None:
            return None
        stop, samples = threading.Event(), []

        def sampler():
            while not stop.is_set():
                samples.append((time.perf_counter(), self.watts(), self.sclk_mhz()))
                stop.wait(0.02)
        th = threading.Thread(target=sampler, daemon=True)
        t0 = time.perf_counter()
        th.start()
        n = 0
        while time.perf_counter() - t0 < seconds:
            for _ in range(10):
                launch()
            torch.cuda.synchronize()
            n += 10
        t1 = time.perf_counter()
        stop.set()
        th.join()
        w_ = [p for t, p, _ in samples if t - t0 >= settle and p is not None]
        f_ = [f for t, _, f in samples if t - t0 >= settle and f is not None]
        if not w_:
            return None
        return {"board_w_mean": round(sum(w_) / len(w_), 1), "board_w_max": round(max(w_), 1),
                "sclk_mhz_mean": round(sum(f_) / len(f_), 0) if f_ else None, "samples": len(w_),
                "launches": n, "ms_per_launch": round((t1 - t0) / n * 1e3, 4)}


def gate_only(args, g, torch) -> int:
    """The memory-bound gate kernels alone, at a size that saturates HBM; algorithmic bytes as in main()
    (the scan-then-propagate variants read their inputs twice: 12 and 20 bytes per element)."""
    B, H, N = (int(x) for x in args.gate_only.split(","))
    gen = torch.Generator(device="cuda:0").manual_seed(1)
    hpre = torch.randn(B, H, N, device="cuda:0", generator=gen) - 1.0
    beta = torch.exp(0.5 * torch.randn(B, H, N, device="cuda:0", generator=gen))
    out1, out2, out3 = torch.empty_like(hpre), torch.empty_like(hpre), torch.empty_like(hpre)
    ws = torch.empty(g.gfwa_gate_scan_workspace_bytes(B, H, N), dtype=torch.uint8, device="cuda:0")
    calls = {
        "gate_prefix_scan": (8.0, lambda: g.gfwa_gate_prefix(hpre, out1)),
        "gate_activation_prefix_scan": (12.0, lambda: g.gfwa_gate_activation_prefix(hpre, beta, args.gate_eps, out1)),
        "gate_activation_bwd": (20.0, lambda: g.gfwa_gate_activation_backward(hpre, beta, args.gate_eps, out1,
                                                                               out2, out3)),
        "gate_prefix_stp": (12.0, lambda: g.gfwa_gate_prefix_stp(hpre, c=out1, workspace=ws)),
        "gate_activation_prefix_stp": (20.0, lambda: g.gfwa_gate_prefix_stp(hpre, beta, args.gate_eps, c=out1, workspace=ws)),
        "plain_copy": (8.0, lambda: out2.copy_(hpre)),
    }
    res = {}
    for name, (bpe, fn) in calls.items():
        for _ in range(args.warmup):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        gbs = bpe * B * H * N / ms / 1e6
        res[name] = {"avg_ms": round(ms, 5), "bytes_per_element": bpe, "achieved": round(gbs, 1), "unit": "GB/s",
                     "peak": PEAK_HBM_GBS, "frac": round(gbs / PEAK_HBM_GBS, 4)}
    print(json.dumps({"metric": "gate kernels, algorithmic GB/s", "shape": [B, H, N], "dtype": "f32",
                      "steps": args.steps, "warmup": args.warmup, "data": "synthetic", "kernels": res}))
    return 0


def decode_only(args, g, torch) -> int:
    """The decoding step alone: HBM-bound on reading the window of the key/value cache once."""
    B, H, Hkv, T, d, w = (int(x) for x in args.decode.split(","))
    dev = "cuda:0"
    gen = torch.Generator(device=dev).manual_seed(2)
    rnd = lambda *shape: torch.randn(*shape, device=dev, generator=gen)
    q = rnd(B, H, d).to(torch.bfloat16)
    Kc, Vc = rnd(B, Hkv, T, d).to(torch.bfloat16), rnd(B, Hkv, T, d).to(torch.bfloat16)
    c = torch.cumsum(torch.nn.functional.softplus(rnd(B, H, T) - 2.0), dim=-1)
    alpha_t = torch.nn.functional.softplus(rnd(B, H) - 2.0)
    pos = torch.full((B,), T - 1, dtype=torch.int32, device=dev)
    o = torch.empty_like(q)
    L = torch.empty(B, H, dtype=torch.float32, device=dev)
    ws = torch.empty(g.gfwa_decode_workspace_bytes(B, H, T, d, w), dtype=torch.uint8, device=dev)
    n = min(w, T)
    # bytes one step has to move: the window of K and V once per key/value head, the window of c once per
    # query head, the query, the output and L
    algo = B * Hkv * n * d * 2 * 2 + B * H * n * 4 + B * H * (2 * d * 2 + 8)

    def step():
        g.gfwa_decode(q, Kc, Vc, c, pos, w, 1.0 / d ** 0.5, alpha_t=alpha_t, o=o, L=L, workspace=ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    g.gfwa_profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) / args.steps * 1e3
    g.gfwa_profile_enable(False)
    prof = {k: v for k, v in g.gfwa_profile_read().items() if v[1]}
    part_ms = prof["decode_partial"][0] / prof["decode_partial"][1]
    comb_ms = prof["decode_combine"][0] / prof["decode_combine"][1] if "decode_combine" in prof else 0.0
    gbs = algo / part_ms / 1e6
    print(json.dumps({
        "metric": "GatedFWA decoding step, algorithmic GB/s of the cache-reading kernel", "value": round(gbs, 1),
        "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(wall_ms, 5),
        "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"decode: B={B} H={H} Hkv={Hkv} T={T} d={d} w={w} bf16 cache, all positions T-1"},
        "roofline": {"kernel": "decode_partial", "bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4), "traffic": None},
        "detail": {"decode_partial_ms": round(part_ms, 5), "decode_combine_ms": round(comb_ms, 5),
                   "algorithmic_bytes": algo, "tokens_per_s": round(B / (wall_ms * 1e-3), 1)}}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # defaults long enough for the clocks to settle: the first ~30 steps after an idle period run up to 30 % slower
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="long_bwd")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--from-preactivation", action="store_true",
                    help="start the step from the gate pre-activation h and amplitude beta instead of alpha: "
                         "fused activation + prefix scan in front, activation backward (dh, dbeta) at the end")
    ap.add_argument("--gate-eps", type=float, default=1e-6)
    ap.add_argument("--gate-only", default=None, metavar="B,H,N",
                    help="time only the memory-bound gate kernels (prefix scan, fused activation + prefix scan, "
                         "gate-gradient scan, activation backward) on [B,H,N] fp32 tensors of this shape, "
                         "e.g. 16,64,262144 (1 GiB per tensor), and print their GB/s instead of the usual line")
    ap.add_argument("--min-workspace", action="store_true",
                    help="give the backward its minimum workspace (the variant that forms S and dP in both passes) "
                         "instead of gfwa_backward_fast_workspace_bytes")
    ap.add_argument("--no-peak-probe", action="store_true", help="skip the pure-MFMA loop and the 1 GiB copy")
    ap.add_argument("--power-pass-seconds", type=float, default=1.0,
                    help="after the timed region: this many seconds of further steps while the board power and the shader "
                         "clock are sampled from the driver's sysfs files (0: skip)")
    ap.add_argument("--power-survey", action="store_true",
                    help="the same sampling also for an idle device, the three MFMA loops, the forward alone and the "
                         "backward alone (about 7 s more)")
    ap.add_argument("--one-pass-prefix", action="store_true",
                    help="always use gfwa_gate_prefix (one workgroup per row) for the prefix, also for few long rows")
    ap.add_argument("--cpu-heads", type=int, default=32)
    ap.add_argument("--traffic-file", default=None,
                    help="text summary of the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs: lines "
                         "'<kernel> <fetch bytes per launch> <write bytes per launch>', '#' comments "
                         "(default: profiles/hbm_traffic_<workload>.txt)")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="before the warm-up, copy this many MiB once with a plain elementwise copy "
                         "kernel (the known-size reference the traffic counters are scaled by)")
    ap.add_argument("--decode", default=None, metavar="B,H,Hkv,T,d,w",
                    help="time the decoding step (one query per head against the cached window, bf16 cache, every "
                         "sequence at position T-1) and print its GB/s on the window's bytes instead of the usual "
                         "line, e.g. 64,32,8,16384,128,1024")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the path has no inter-GPU part); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import gfwa_inputs as gi
    import paper_2512_07782_amd as g

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    g.load_library()
    dev = "cuda:0"
    if args.gate_only:
        return gate_only(args, g, torch)
    if args.decode:
        return decode_only(args, g, torch)
    wl = gi.WORKLOADS[args.workload]
    ins = {t: gi.make_tensor(wl, t) for t in ("Q", "K", "V", "alpha", "dO")} if wl.backward else gi.make_inputs(wl)
    bf = wl.dtype == "bf16"
    peak_tf, peak_name = (PEAK_BF16_TFLOPS, "bf16") if bf else (PEAK_F32_TFLOPS, "f32")   # the matrix cores the workload's kernels use
    to = lambda x, b: (torch.from_numpy(x).to(dev).to(torch.bfloat16) if b else torch.from_numpy(x).to(dev))
    Q, K, V = (to(ins[k], bf) for k in ("Q", "K", "V"))
    dO = to(ins["dO"], bf) if wl.backward else None
    alpha = to(ins["alpha"], False)
    B, H, N, d, w = wl.B, wl.H, wl.N, wl.d, wl.w

    if args.from_preactivation:
        hpre, beta = (to(x, False) for x in gi.make_gate_inputs(wl))
        dh, dbeta = torch.empty_like(hpre), torch.empty_like(hpre)
    c = torch.empty_like(alpha)
    O = torch.empty_like(Q)
    L = torch.empty((B, H, N), dtype=torch.float32, device=dev)
    if wl.backward:
        dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
        dalpha = torch.empty_like(alpha)
        ws_size = g.gfwa_backward_workspace_bytes if args.min_workspace else g.gfwa_backward_fast_workspace_bytes
        ws = torch.empty(ws_size(Q.dtype, B, H, N, d, w), dtype=torch.uint8, device=dev)

    gqa = wl.Hkv != wl.H   # grouped-query workloads go through the entry points that take [B,Hkv,N,d] keys
    fwd, bwd = (g.gfwa_forward_gqa, g.gfwa_backward_gqa) if gqa else (g.gfwa_forward, g.gfwa_backward)

    # few long rows: the caller picks the scan-then-propagate form of the prefix (one workgroup per row would
    # leave most of the chip idle); the backward's gradient scan makes the same choice inside the library
    ncu = torch.cuda.get_device_properties(0).multi_processor_count
    stp = (B * H < ncu and N >= 8192) and not args.one_pass_prefix
    stp_ws = torch.empty(g.gfwa_gate_scan_workspace_bytes(B, H, N), dtype=torch.uint8, device=dev) if stp else None

    def prefix():
        if args.from_preactivation:
            if stp:
                g.gfwa_gate_prefix_stp(hpre, beta, args.gate_eps, c=c, workspace=stp_ws)
            else:
                g.gfwa_gate_activation_prefix(hpre, beta, args.gate_eps, c)
        elif stp:
            g.gfwa_gate_prefix_stp(alpha, c=c, workspace=stp_ws)
        else:
            g.gfwa_gate_prefix(alpha, c)

    def step():
        prefix()
        fwd(Q, K, V, c, w, wl.scale, O=O, L=L)
        if wl.backward:
            bwd(Q, K, V, O, dO, c, L, w, wl.scale, workspace=ws, dQ=dQ, dK=dK, dV=dV, dalpha=dalpha)
            if args.from_preactivation:
                g.gfwa_gate_activation_backward(hpre, beta, args.gate_eps, dalpha, dh, dbeta)

    if args.copy_calibration_mib > 0:
        src = torch.ones(args.copy_calibration_mib << 18, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- what this device sustains: bf16 MFMA loops on every SIMD, and a plain 1 GiB copy.  Run first: about a third of
    # a second of load (the copy first, the matrix-core loops last, so that what follows starts on a part under load)
    achievable = None
    if not args.no_peak_probe:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        sink = torch.zeros(1, dtype=torch.float32, device=dev)
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        best_gb = 0.0
        for rep in range(4):
            e0.record()
            nbytes = g.gfwa_probe_copy(src, dst)
            e1.record()
            torch.cuda.synchronize()
            if rep:
                best_gb = max(best_gb, 2.0 * nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9)
        del src, dst
        best = {0: 0.0, 1: 0.0, 2: 0.0}
        for random_operands in (0, 1, 2):
            for rep in range(4):   # the first repetition also settles the clock under this load
                e0.record()
                flops = g.gfwa_probe_mfma(sink, 40000, ncu, random_operands)
                e1.record()
                torch.cuda.synchronize()
                if rep:
                    best[random_operands] = max(best[random_operands], flops / (e0.elapsed_time(e1) * 1e-3) / 1e12)
        best_tf, best_tf_random, best_tf_mix = best[0], best[1], best[2]
        achievable = {"mfma_bf16_tflops": round(best_tf, 1), "mfma_frac_of_published": round(best_tf / PEAK_BF16_TFLOPS, 4),
                      "mfma_bf16_tflops_random_operands": round(best_tf_random, 1),
                      "mfma_random_frac_of_published": round(best_tf_random / PEAK_BF16_TFLOPS, 4),
                      "mfma_bf16_tflops_attention_mix": round(best_tf_mix, 1),
                      "mfma_mix_frac_of_published": round(best_tf_mix / PEAK_BF16_TFLOPS, 4),
                      "copy_gbs": round(best_gb, 1), "copy_frac_of_published": round(best_gb / PEAK_HBM_GBS, 4),
                      "how": "gfwa_probe_mfma: 40000 x 16 MFMAs per wave, 8 waves on every CU, best of 3, once with one "
                             "constant operand pair, once with sixteen pseudo-random unit-variance pairs (the clock "
                             "the part sustains depends on how much the operands switch), once with those and one LDS "
                             "fragment read, four fma and one exp2 per MFMA (the least an attention inner loop does); "
                             "gfwa_probe_copy: 1 GiB read + 1 GiB written, best of 3"}

    # ---- the breakdown pass, in front of the timed region: the same steps with one HIP event between the calls of a
    # step (per-call and per-step durations -> median, min) and the library's event pair around every kernel launch.
    # After any change of load the part takes about 25 steps (30 ms) to settle its clocks - also after the
    # calibration loops above - so this pass doubles as the run-in that lets a short timed region see the steady state.
    for _ in range(args.warmup):
        step()
    marks = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    g.gfwa_profile_enable(True)
    for k in range(args.steps):
        marks[k][0].record()
        prefix()
        marks[k][1].record()
        fwd(Q, K, V, c, w, wl.scale, O=O, L=L)
        marks[k][2].record()
        if wl.backward:
            bwd(Q, K, V, O, dO, c, L, w, wl.scale, workspace=ws, dQ=dQ, dK=dK, dV=dV, dalpha=dalpha)
            if args.from_preactivation:
                g.gfwa_gate_activation_backward(hpre, beta, args.gate_eps, dalpha, dh, dbeta)
        marks[k][3].record()
    torch.cuda.synchronize()
    g.gfwa_profile_enable(False)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # ---- the timed region: exactly `steps` steps, nothing else on the stream, wall clock
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3

    prof = g.gfwa_profile_read()

    # ---- after the timed region: what the board draws while the same steps keep running
    power = None
    if args.power_pass_seconds > 0:
        bp = BoardPower(torch)
        power = bp.during(torch, step, args.power_pass_seconds)
        if power is not None:
            power["cap_w"] = bp.cap_watts()
            power["how"] = (f"{args.power_pass_seconds:g} s of further steps after the timed region; hwmon power1_input and the "
                            "active pp_dpm_sclk level sampled every 20 ms, the first 0.3 s dropped")
            if args.power_survey:
                sink = torch.zeros(1, dtype=torch.float32, device=dev)
                secs = args.power_pass_seconds
                survey = {"idle": bp.during(torch, lambda: time.sleep(0.005), secs)}
                for mode, name in ((0, "mfma_constant_operands"), (1, "mfma_random_operands"), (2, "mfma_attention_mix")):
                    survey[name] = bp.during(torch, lambda: g.gfwa_probe_mfma(sink, 2000, ncu, mode), secs)
                survey["forward"] = bp.during(torch, lambda: fwd(Q, K, V, c, w, wl.scale, O=O, L=L), secs)
                if wl.backward:
                    survey["backward"] = bp.during(torch, lambda: bwd(Q, K, V, O, dO, c, L, w, wl.scale, workspace=ws, dQ=dQ,
                                                                      dK=dK, dV=dV, dalpha=dalpha), secs)
                power["survey"] = survey

    def stats(xs):
        xs = sorted(xs)
        return {"avg": round(sum(xs) / len(xs), 5), "median": round(xs[len(xs) // 2], 5), "min": round(xs[0], 5)}
    call_ms = {
        "gate_prefix": stats([m[0].elapsed_time(m[1]) for m in marks]),
        "forward": stats([m[1].elapsed_time(m[2]) for m in marks]),
        "step": stats([a[0].elapsed_time(b[0]) for a, b in zip(marks[:-1], marks[1:])] or [marks[0][0].elapsed_time(marks[0][3])]),
    }
    if wl.backward:
        call_ms["backward"] = stats([m[2].elapsed_time(m[3]) for m in marks])

    f_fwd = wl.flops_fwd_nominal()
    f_bwd = wl.flops_bwd_nominal() if wl.backward else 0.0
    bhn = B * H * N
    # algorithmic work per launch of each kernel
    algo = {
        "gate_prefix_scan": ("hbm", 8.0 * bhn),
        "forward": ("mfma", f_fwd),
        "bwd_rowdot": ("hbm", bhn * (4.0 * d + 4.0)),
        "bwd_dkv": ("mfma", 8.0 * bhn * w * d),     # S, dP, dV, dK products
        "bwd_dq": ("mfma", 2.0 * bhn * w * d),      # the dQ product; its S and dP are recomputation (bf16: also forms D)
        "gate_grad_scan": ("hbm", 12.0 * bhn),
        "gate_activation_prefix_scan": ("hbm", 12.0 * bhn),   # h, beta in; c out
        "gate_activation_bwd": ("hbm", 20.0 * bhn),           # h, beta, dalpha in; dh, dbeta out
        # a scan cut into segments is two launches, the first reading the inputs once more
        "scan_segment_sum": ("hbm", (8.0 if args.from_preactivation else 4.0) * bhn),
        "scan_propagate": ("hbm", (12.0 if args.from_preactivation else 8.0) * bhn),
        "gate_grad_segment_sum": ("hbm", 8.0 * bhn),
    }
    kernels = {}
    for name, (tot, cnt) in prof.items():
        if cnt == 0:
            continue
        avg_ms = tot / cnt
        bound, work = algo[name]
        if bound == "mfma":
            ach, peak, unit = work / (avg_ms * 1e-3) / 1e12, peak_tf, "TFLOP/s"
        else:
            ach, peak, unit = work / (avg_ms * 1e-3) / 1e9, PEAK_HBM_GBS, "GB/s"
        kernels[name] = {"avg_ms": round(avg_ms, 5), "launches": cnt, "bound": bound, "achieved": round(ach, 2),
                         "peak": peak, "unit": unit, "frac": round(ach / peak, 4)}
    dominant = max(kernels, key=lambda k: kernels[k]["avg_ms"])
    # measured HBM bytes per launch (fetch + write) of the dominant kernel, from the counter runs
    traffic = None
    # (the committed summary is of the default run: the backward with its dS-block workspace)
    tfile = args.traffic_file or os.path.join(ROOT, "profiles", f"hbm_traffic_{args.workload}"
                                              + ("_min_workspace" if args.min_workspace else "") + ".txt")
    if os.path.exists(tfile):
        for line in open(tfile):
            f = line.split("#")[0].split()
            if len(f) == 3 and f[0] == dominant:
                traffic = float(f[1]) + float(f[2])
    roofline = {"kernel": dominant, "bound": kernels[dominant]["bound"], "achieved": kernels[dominant]["achieved"],
                "peak": kernels[dominant]["peak"], "unit": kernels[dominant]["unit"],
                "frac": kernels[dominant]["frac"], "traffic": traffic,
                "traffic_source": (os.path.relpath(tfile, ROOT) + " (rocprofv3 --pmc runs of this command, committed; not "
                                   "measured in this run)") if traffic is not None else None}

    fwd_ms = call_ms["forward"]["avg"]
    detail = {"fwd_ms": fwd_ms, "fwd_ms_median": call_ms["forward"]["median"], "fwd_ms_min": call_ms["forward"]["min"],
              "fwd_tflops_nominal": round(f_fwd / fwd_ms / 1e9, 2),
              "fwd_tflops_exact": round(wl.flops_fwd_exact() / fwd_ms / 1e9, 2),
              f"fwd_frac_{peak_name}_peak": round(f_fwd / fwd_ms / 1e9 / peak_tf, 4)}
    if wl.backward:
        bwd_ms = call_ms["backward"]["avg"]
        detail.update({"bwd_ms": round(bwd_ms, 5), "bwd_ms_median": call_ms["backward"]["median"],
                       "bwd_ms_min": call_ms["backward"]["min"], "bwd_tflops_nominal": round(f_bwd / bwd_ms / 1e9, 2),
                       f"bwd_frac_{peak_name}_peak": round(f_bwd / bwd_ms / 1e9 / peak_tf, 4)})
    detail["step_ms_median"] = call_ms["step"]["median"]
    detail["step_ms_min"] = call_ms["step"]["min"]
    detail["gate_prefix_ms"] = call_ms["gate_prefix"]["avg"]
    detail["timing"] = ("ms_per_step and value: wall clock over the timed region (steps only); fwd_ms, bwd_ms, gate_prefix_ms "
                        "and the medians/minima: one HIP event between the calls of a step, in a pass of the same steps "
                        "(after its own warm-up steps) that runs before the warm-up and the timed region and so also "
                        "serves as run-in: the part needs about 25 steps to settle after a change of load; kernels.*: "
                        "the library's event pair around every launch in that pass (a few microseconds of overhead "
                        "each, visible on the ~10 us scans)")
    if power is not None:
        detail["power"] = power
    if achievable and bf:   # the probes are bf16 loops
        detail["fwd_frac_of_achievable_mfma"] = round(f_fwd / fwd_ms / 1e9 / achievable["mfma_bf16_tflops"], 4)
        detail["fwd_frac_of_achievable_mfma_random_operands"] = round(
            f_fwd / fwd_ms / 1e9 / achievable["mfma_bf16_tflops_random_operands"], 4)
        if wl.backward:
            detail["bwd_frac_of_achievable_mfma"] = round(f_bwd / bwd_ms / 1e9 / achievable["mfma_bf16_tflops"], 4)
            detail["bwd_frac_of_achievable_mfma_random_operands"] = round(
                f_bwd / bwd_ms / 1e9 / achievable["mfma_bf16_tflops_random_operands"], 4)

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        G = H // wl.Hkv
        nh = max(G, min(args.cpu_heads, B * H) // G * G)     # whole groups
        heads = list(range(nh))
        sel = lambda x, tr: oracle.select_heads(x, heads, tr)
        # the first nh query heads and the nh / G key/value heads they read, as one batch entry
        selq = lambda x: sel(x, 2).reshape(1, nh, N, d)
        selk = lambda x: oracle.select_heads(x, list(range(nh // G)), 2).reshape(1, nh // G, N, d)
        t0 = time.perf_counter()
        if args.from_preactivation:
            hb = [sel(x, 1) for x in gi.make_gate_inputs(wl)]
            cs = oracle.gate_prefix(oracle.gate_activation(hb[0], hb[1], args.gate_eps))
        else:
            cs = oracle.gate_prefix(sel(ins["alpha"], 1))
        fw = gr = None
        if wl.backward:
            gr = oracle.backward_gqa_from_c(selq(ins["Q"]), selk(ins["K"]), selk(ins["V"]), cs.reshape(1, nh, N),
                                            selq(ins["dO"]), w, wl.scale)
            if args.from_preactivation:
                oracle.gate_activation_backward(hb[0], hb[1], args.gate_eps, gr["dalpha"].reshape(hb[0].shape))
        else:
            fw = oracle.forward_gqa_from_c(selq(ins["Q"]), selk(ins["K"]), selk(ins["V"]), cs.reshape(1, nh, N), w, wl.scale)
        dt_cpu = time.perf_counter() - t0
        frac = nh / (B * H)
        cpu = {"value": round((f_fwd + f_bwd) * frac / dt_cpu / 1e12, 5), "unit": "TFLOP/s", "cores": oracle.threads(),
               "kind": "oracle", "sample": f"{nh} of {B*H} (b,h) heads of the same workload, forward"
               + ("+backward" if wl.backward else "") + f", {dt_cpu:.1f} s"}
        # parity of the very tensors the timed steps left behind, on the heads the oracle just computed (after the
        # timed oracle work above: the forward of the same heads once more for O and L)
        hostf = lambda t_: t_.detach().to(torch.float32).cpu().numpy().astype(np.float64)
        if fw is None:
            fw = oracle.forward_gqa_from_c(selq(ins["Q"]), selk(ins["K"]), selk(ins["V"]), cs.reshape(1, nh, N), w, wl.scale)
        O_ref, L_ref = fw
        errO = np.abs(selq(hostf(O)) - O_ref)
        par = {"heads": nh, "c_max_rel": float(np.abs(sel(hostf(c), 1) - cs).max() / cs.max()),
               "O_max_abs": float(errO.max()), "O_mean_abs": float(errO.mean()),
               "L_max_abs": float(np.abs(sel(hostf(L), 1).reshape(1, nh, N) - L_ref).max())}
        if gr is not None:
            rel = lambda a_, r_: float(np.linalg.norm((a_ - r_).ravel()) / max(np.linalg.norm(r_.ravel()), 1e-300))
            par.update({"dQ_rel_l2": rel(selq(hostf(dQ)), gr["dQ"]), "dK_rel_l2": rel(selk(hostf(dK)), gr["dK"]),
                        "dV_rel_l2": rel(selk(hostf(dV)), gr["dV"]),
                        "dalpha_rel_l2": rel(sel(hostf(dalpha), 1).reshape(1, nh, N), gr["dalpha"])})
        par = {k: (round(v, 10) if isinstance(v, float) else v) for k, v in par.items()}
        if bf:
            bars = {"O_max_abs": 2e-2, "O_mean_abs": 2e-3, "dQ_rel_l2": 1e-2, "dK_rel_l2": 1e-2, "dV_rel_l2": 1e-2, "dalpha_rel_l2": 1e-2}
        else:
            # fp32 storage: 1e-5 relative on equal inputs.  Here the inputs are not quite equal: the timed step forms
            # its own fp32 prefix c, the oracle an fp64 one, and a logit holds a difference of two c - so the bar
            # carries the rounding of c on top (2 ulp of its largest value, as a relative error of a probability)
            par["O_rel_inf"] = round(float(errO.max() / np.abs(O_ref).max()), 10)
            par["L_rel_inf"] = round(float(par["L_max_abs"] / np.abs(L_ref).max()), 10)
            bar = 1e-5 + 2.0 * 2.0 ** -24 * float(cs.max())
            par["fp32_bar"] = round(bar, 10)
            bars = {k: bar for k in ("O_rel_inf", "L_rel_inf", "dQ_rel_l2", "dK_rel_l2", "dV_rel_l2", "dalpha_rel_l2")}
        # (the literal bars are for unit-variance values; the gate-extreme workload has its own, derived ones)
        par["within_stated_tolerances"] = bool(all(par[k] <= bars[k] for k in bars if k in par)) if wl.qkv_std == 1.0 else None
        detail["parity"] = par

    out = {
        "metric": "GatedFWA fwd+bwd effective TFLOP/s (in-window FLOPs, nominal) on 1 GPU",
        "value": round((f_fwd + f_bwd) / (ms_per_step * 1e-3) / 1e12, 2),
        "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: B={B} H={H}" + (f" Hkv={wl.Hkv}" if gqa else "") + f" N={N} d={d} w={w} {wl.dtype}, "
                   + ("gate activation + prefix" if args.from_preactivation else "gate prefix") + " + forward"
                   + (" + backward" if wl.backward else "")
                   + (" + gate activation backward" if args.from_preactivation and wl.backward else ""), f"peak_{peak_name}_tflops": peak_tf,
                   "backward_workspace_mb": round(ws.numel() / 1e6, 1) if wl.backward else None,
                   "gate_prefix": "scan-then-propagate (few long rows)" if stp else "one pass"},
        "roofline": roofline, "cpu_baseline": cpu, "achievable": achievable, "detail": detail, "kernels": kernels,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
