"""The JSON line of bench.py, produced in this process on the GPU (a short run of a small workload and of the
default one): the keys and types the measurement contract names, and that the figures are consistent with
each other."""
import json
import sys

import pytest

import bench
import gfwa_inputs as gi

pytestmark = pytest.mark.gpu


def _run(monkeypatch, capsys, *argv):
    monkeypatch.setattr(sys, "argv", ["bench.py", *argv])
    assert bench.main() == 0
    lines = [l for l in capsys.readouterr().out.splitlines() if l.startswith("{")]
    assert len(lines) == 1, "exactly one JSON line"
    return json.loads(lines[0])


def _check_common(d, steps, warmup, dtype="bf16"):
    assert d["n_gpus"] == 1 and d["steps"] == steps and d["warmup"] == warmup
    assert d["higher_is_better"] is True and d["scaling"] == "weak" and d["data"] == "synthetic"
    assert d["unit"] == "TFLOP/s" and d["dtype"] == dtype and d["vs_baseline"] is None
    assert isinstance(d["config"]["workload"], str) and "model" not in d["config"]
    assert d["value"] > 0 and d["ms_per_step"] > 0
    r = d["roofline"]
    assert r["bound"] in ("hbm", "mfma", "alu") and r["unit"] in ("GB/s", "TFLOP/s")
    assert r["peak"] > 0 and abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3
    assert "traffic" in r


def test_small_workload_with_oracle_baseline(monkeypatch, capsys):
    d = _run(monkeypatch, capsys, "--workload", "lm_gqa_bwd", "--steps", "3", "--warmup", "1", "--no-peak-probe",
             "--power-pass-seconds", "0.4", "--cpu-heads", "4")
    _check_common(d, 3, 1)
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["value"] > 0 and c["cores"] >= 1 and isinstance(c["sample"], str)
    par = d["detail"]["parity"]
    assert par["within_stated_tolerances"] is True and par["heads"] == 4
    # whole-step throughput follows from the nominal FLOP count and the wall time
    wl = gi.WORKLOADS["lm_gqa_bwd"]
    tf = (wl.flops_fwd_nominal() + wl.flops_bwd_nominal()) / (d["ms_per_step"] * 1e-3) / 1e12
    assert abs(tf - d["value"]) <= 0.02 * d["value"]
    p = d["detail"].get("power")
    if p is not None:   # present wherever the driver exposes the sensors
        assert 0 < p["board_w_mean"] <= p["board_w_max"] and p["samples"] >= 1


def test_default_workload_short(monkeypatch, capsys):
    d = _run(monkeypatch, capsys, "--steps", "3", "--warmup", "1", "--no-cpu-baseline", "--power-pass-seconds", "0")
    _check_common(d, 3, 1)
    assert d["config"]["workload"].startswith("long_bwd") and d["cpu_baseline"] is None
    assert d["roofline"]["kernel"] == "bwd_dkv" and d["roofline"]["bound"] == "mfma" and d["roofline"]["peak"] == 2500.0
    a = d["achievable"]
    assert a["mfma_bf16_tflops"] > a["mfma_bf16_tflops_random_operands"] > a["mfma_bf16_tflops_attention_mix"] > 0
    assert a["copy_gbs"] > 0
    k = d["kernels"]
    for name in ("forward", "bwd_rowdot", "bwd_dkv", "bwd_dq"):
        assert k[name]["launches"] == 3 and k[name]["avg_ms"] > 0


def test_fp32_workload_is_priced_against_the_fp32_peak(monkeypatch, capsys):
    d = _run(monkeypatch, capsys, "--workload", "mid_bwd_f32", "--steps", "2", "--warmup", "1", "--no-peak-probe",
             "--power-pass-seconds", "0", "--cpu-heads", "2")
    _check_common(d, 2, 1, dtype="f32")
    assert d["roofline"]["bound"] == "mfma" and d["roofline"]["peak"] == 157.3
    assert 0 < d["detail"]["fwd_frac_f32_peak"] < 1 and 0 < d["detail"]["bwd_frac_f32_peak"] < 1
    par = d["detail"]["parity"]
    assert par["within_stated_tolerances"] is True and par["O_rel_inf"] <= par["fp32_bar"] < 1e-3
