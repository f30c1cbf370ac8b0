"""bench.py on a GPU: the one JSON line it prints carries the fields the benchmark contract names,
its figures are consistent with each other, and the modes beside the headline still run."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                       timeout=300, cwd=ROOT)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [ln for ln in p.stdout.splitlines() if ln.startswith("{")]
    assert len(lines) == 1, p.stdout[-2000:]
    return json.loads(lines[0])


def test_headline_line_of_a_mid_sized_workload():
    r = _run("--config", "2", "--steps", "30", "--warmup", "5", "--no-all-configs")
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in r, key
    assert r["n_gpus"] == 1 and r["steps"] == 30 and r["warmup"] == 5 and r["vs_baseline"] is None
    assert r["dtype"] == "f32" and r["logits_dtype"] == "bf16" and r["data"] == "synthetic"
    assert r["config"]["workload"].startswith("cfg2") and "model" not in r["config"]
    assert abs(r["value"] - r["config"]["draft_positions"] / (r["ms_per_step"] * 1e-3)) < 1e-6 * r["value"]
    roof = r["roofline"]
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-9
    assert abs(roof["achieved"] - roof["algorithmic_bytes_per_launch"] / (roof["avg_launch_us"] * 1e-6) / 1e9) < 1e-6 * roof["achieved"]
    assert roof["algorithmic_bytes_per_launch"] == 2304 * 128256 * 2
    assert 0.3 < roof["frac"] < 1.0                                  # a statistics kernel that streams
    assert roof["avg_launch_us"] * 1e-3 < r["ms_per_step"]           # the dominant kernel fits inside the step
    assert roof["frac_of_measured_read_ceiling"] <= 1.0              # the probe sweep is a ceiling
    rm = r["resid_mass_roofline"]                                    # cfg2: 242 rejected sessions
    assert abs(rm["algorithmic_bytes_per_launch"] - rm["rejected_sessions_per_launch"] * 128256 * 6) < 1.0
    assert 0.5 * 256 < rm["rejected_sessions_per_launch"] <= 256 and 0 < r["config"]["rejected_sessions"] <= 256
    assert 0.2 < rm["frac"] < 1.0 and rm["frac_of_measured_read_ceiling"] <= 1.0
    ev = r["step_events"]
    assert ev["min_ms"] <= ev["median_ms"] <= ev["max_ms"]
    cpu = r["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] == 1 and cpu["value"] > 0 and "sample" in cpu
    assert r["whole_step_call"]["ms_per_step"] > 0 and r["early_exit_mode"]["ms_per_step"] > 0


def test_all_configs_block_and_small_modes():
    r = _run("--config", "1", "--steps", "50", "--warmup", "5", "--no-cpu-baseline")
    assert set(r["all_configs"]) == {f"cfg{i}" for i in range(5)}
    for name, c in r["all_configs"].items():
        assert c["three_calls"]["ms_per_step"] > 0 and c["whole_step_call"]["ms_per_step"] > 0, name
        assert c["three_calls"]["events"]["median_ms"] > 0, name
    assert r["all_configs"]["cfg4"]["row_chunk_stats"]["frac_of_hbm_peak"] > 0.5
    for extra in (("--fused",), ("--early-exit", "--fused"), ("--split",), ("--top-k", "10"), ("--graph",),
                  ("--rotate", "3")):
        q = _run("--config", "1", "--steps", "20", "--warmup", "3", "--no-cpu-baseline", "--no-all-configs", *extra)
        assert q["value"] > 0 and q["ms_per_step"] > 0, extra


def test_more_steps_than_the_library_has_timing_brackets():
    """The library keeps 2048 event pairs per kernel: a longer run brackets its first steps only
    and still times all of them by the wall clock."""
    r = _run("--config", "0", "--steps", "2500", "--warmup", "5", "--no-cpu-baseline", "--no-all-configs",
             "--headline-only")
    assert r["steps"] == 2500 and r["value"] > 0 and r["roofline"]["avg_launch_us"] > 0
    q = _run("--config", "2", "--steps", "300", "--warmup", "5", "--no-cpu-baseline", "--no-all-configs",
             "--early-exit", "--fused")
    assert q["steps"] == 300 and q["value"] > 0 and q["roofline"]["avg_launch_us"] > 0


def test_copy_probe_line():
    r = _run("--copy-probe")
    assert r["copy_probe"] and r["bytes_read_per_launch"] == 2 << 30 and r["GBps_read_plus_write"] > 1000
