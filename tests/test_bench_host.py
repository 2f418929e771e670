"""Host-side pieces of bench.py that need no GPU: the sysfs clock/power sampler and the refusal of more than one GPU."""
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def _fake_sysfs(tmp_path, current="1: 1891Mhz *"):
    dev = tmp_path / "card0" / "device"
    hw = dev / "hwmon" / "hwmon3"
    hw.mkdir(parents=True)
    (dev / "pp_dpm_sclk").write_text(f"0: 500Mhz\n{current}\n2: 2400Mhz\n")
    (hw / "power1_input").write_text("1315000000\n")
    (hw / "power1_cap").write_text("1400000000\n")
    (hw / "temp2_input").write_text("55000\n")
    (hw / "temp3_input").write_text("61000\n")
    return str(tmp_path)


def test_sampler_reads_clock_power_and_temperature(tmp_path):
    s = bench.EngineClockSampler(_fake_sysfs(tmp_path))
    assert s.max_mhz == 2400.0 and s.power_cap_w == 1400.0
    with s:
        time.sleep(0.1)
    r = s.summary()
    assert r["samples"] >= 2
    assert r["engine_clock_mhz_median"] == r["engine_clock_mhz_min"] == r["engine_clock_mhz_max"] == 1891.0
    assert r["power_w_median"] == 1315.0 and r["hottest_sensor_c_median"] == 61.0


def test_sampler_without_sysfs_reports_nothing(tmp_path):
    s = bench.EngineClockSampler(str(tmp_path / "absent"))
    with s:
        pass
    r = s.summary()
    assert r["samples"] == 0 and r["engine_clock_mhz_median"] is None and r["power_cap_w"] is None
    assert s.max_mhz is None


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)
