"""The benchmark's command line and output line: the keys a consumer relies on."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args, timeout=300):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, capture_output=True,
                          text=True, timeout=timeout)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run_bench("--gpus", "2")
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)


@pytest.mark.gpu
def test_default_workload_line_has_the_contract_keys():
    r = run_bench("--steps", "20", "--warmup", "5", "--no-cpu-baseline")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.startswith("{")]
    assert len(lines) == 1
    out = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "staged"):
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == 20 and out["warmup"] == 5
    assert out["unit"] == "GB/s" and out["higher_is_better"] is True and out["vs_baseline"] is None
    assert out["data"] == "synthetic" and out["config"]["workload"] == "llama8b_boundary"
    rf = out["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and rf["unit"] == "GB/s"
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3
    assert rf["traffic"] is None or rf["traffic"] >= rf["bytes_per_launch"]
    assert rf["plain_copy"]["bytes_read_plus_written"] == rf["bytes_per_launch"] and rf["plain_copy"]["gbps"] > 0
    # whole-step throughput cannot exceed what the launches achieve back to back
    assert 0 < out["value"] <= rf["achieved"] * 1.02
    st = out["staged"]
    assert 0 < st["round_trip_gbps"] <= min(st["probe_d2h_gbps"], st["probe_h2d_gbps"])


@pytest.mark.gpu
def test_stream_workload_line():
    r = run_bench("--workload", "stream_1f1b", "--steps", "5", "--warmup", "2")
    assert r.returncode == 0, r.stderr[-2000:]
    out = json.loads([ln for ln in r.stdout.splitlines() if ln.startswith("{")][-1])
    assert out["config"]["workload"] == "stream_1f1b" and out["value"] > 0 and out["us_per_micro_batch"] > 0
