"""Host-side parts of bench.py that need no GPU: the reader of the driver's power and clock files, and the
refusal of more than one GPU."""
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


class _NoGpu:
    """Stands in for torch: no device properties (the single card found is taken), synchronize does nothing."""
    class cuda:
        @staticmethod
        def get_device_properties(i):
            raise RuntimeError("no device")

        @staticmethod
        def synchronize():
            pass


def _fake_card(tmp_path, power="1397000000", cap="1400000000", sclk="0: 500Mhz\n1: 1912Mhz *\n2: 2400Mhz\n"):
    hw = tmp_path / "card0" / "device" / "hwmon" / "hwmon3"
    hw.mkdir(parents=True)
    (hw / "power1_input").write_text(power)
    (hw / "power1_cap").write_text(cap)
    (tmp_path / "card0" / "device" / "pp_dpm_sclk").write_text(sclk)
    return str(tmp_path)


def test_board_power_reads_the_files(tmp_path):
    bp = bench.BoardPower(_NoGpu, sysfs=_fake_card(tmp_path))
    assert bp.watts() == 1397.0
    assert bp.cap_watts() == 1400.0
    assert bp.sclk_mhz() == 1912.0


def test_board_power_sampling(tmp_path):
    bp = bench.BoardPower(_NoGpu, sysfs=_fake_card(tmp_path))
    calls = []

    def launch():   # like a GPU launch it lets go of the interpreter, so that the sampling thread gets its turns
        calls.append(1)
        time.sleep(0.001)
    r = bp.during(_NoGpu, launch, seconds=0.4, settle=0.05)
    assert r["board_w_mean"] == 1397.0 and r["board_w_max"] == 1397.0 and r["sclk_mhz_mean"] == 1912.0
    assert r["samples"] >= 1 and r["launches"] == len(calls) and r["launches"] % 10 == 0


def test_board_power_absent(tmp_path):
    bp = bench.BoardPower(_NoGpu, sysfs=str(tmp_path))          # no card at all
    assert bp.watts() is None and bp.cap_watts() is None and bp.sclk_mhz() is None
    assert bp.during(_NoGpu, lambda: None, seconds=0.05) is None
    bp = bench.BoardPower(_NoGpu, sysfs=_fake_card(tmp_path, power="N/A", sclk="garbage"))
    assert bp.watts() is None and bp.sclk_mhz() is None


def test_more_than_one_gpu_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0
    assert "one GPU" in (p.stdout + p.stderr)
