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


def test_traffic_figure_is_readable_for_this_build():
    """roofline.traffic comes from the tracked counter summary: its `library:` line must name the version this
    source tree builds (the line would otherwise carry null without anybody noticing)."""
    sys.path.insert(0, ROOT)
    import bench
    from paper_2602_18007_amd import hxt
    got = bench.traffic_from_profile(hxt.hxt_version())
    assert isinstance(got, int) and got >= 4 * 33554432
    assert bench.traffic_from_profile("some other build") is None


def one_line(r):
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.startswith("{")]
    assert len(lines) == 1
    return json.loads(lines[0])


def check_contract(out, steps, warmup):
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "repeats", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "staged", "regions"):
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == steps and out["warmup"] == warmup and out["repeats"] >= 5
    assert out["unit"] == "GB/s" and out["higher_is_better"] is True and out["vs_baseline"] is None
    assert out["data"] == "synthetic" and out["config"]["workload"] == "llama8b_boundary"
    assert out["value_region"] == "chains_cold" and out["value"] == out["regions"]["chains_cold"]["gbps"]
    assert "all-cold" in out["config"]["cache_state"]
    rf = out["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and rf["unit"] == "GB/s" and rf["region"] == "cold"
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3
    assert isinstance(rf["traffic"], int) and rf["traffic"] >= rf["bytes_per_launch"]
    assert rf["plain_copy"]["bytes_read_plus_written"] == rf["bytes_per_launch"] and rf["plain_copy"]["gbps"] > 0
    # one stream: whole-region throughput cannot exceed what the launches achieve back to back
    assert 0 < out["regions"]["cold"]["gbps"] <= rf["achieved"] * 1.02
    assert 0 < out["value"] < rf["peak"]
    # the timed region is long enough that one synchronisation does not show
    assert out["regions"]["cold"]["timed_steps"] == steps * out["repeats"] and out["regions"]["cold"]["wall_ms"] > 20
    assert out["regions"]["chains_cold"]["timed_steps"] == steps * out["repeats"]
    for name in ("llc", "chains_cold", "chains_llc"):
        assert out["regions"][name]["gbps"] > 0
    st = out["staged"]
    assert 0 < st["round_trip_gbps"] <= min(st["probe_d2h_gbps"], st["probe_h2d_gbps"])
    assert 50 < st["bound_pct"] <= 100


@pytest.mark.gpu
def test_default_workload_line_has_the_contract_keys():
    out = one_line(run_bench("--steps", "20", "--warmup", "5", "--no-cpu-baseline", "--no-configs"))
    check_contract(out, 20, 5)


@pytest.mark.gpu
def test_default_run_lists_every_benchmark_message():
    out = one_line(run_bench("--steps", "20", "--warmup", "5", timeout=900))
    check_contract(out, 20, 5)
    cb = out["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] >= 1 and cb["value"] > 0 and cb["sample"]
    names = {(e["workload"], e["path"]) for e in out["configs"]}
    for want in (("tiny", "device_direct"), ("llama8b_boundary", "device_direct"), ("qwen2_7b_boundary", "device_direct"),
                 ("qwen2_7b_boundary", "cpu_forward"), ("stream_1f1b", "device_direct"), ("stream_1f1b", "cpu_forward"),
                 ("grad_buckets", "device_direct"), ("grad_buckets", "cpu_forward"), ("qwen_rows_view", "device_direct"),
                 ("transpose_view", "device_direct"), ("rows_split_view", "device_direct"),
                 ("inner_stride_view", "device_direct"), ("wide_transpose_view", "device_direct")):
        assert want in names, want
    for e in out["configs"]:
        if e["path"] == "device_direct":
            assert e["gbps"] > 0 and 0 < e["pct_hbm_peak"] < 100
        else:
            assert 0 < e["pct_host_link"] <= 100 and 50 < e["bound_pct"] <= 100
        assert e["cpu_oracle_gbps"] > 0


@pytest.mark.gpu
def test_stream_workload_line():
    out = one_line(run_bench("--workload", "stream_1f1b", "--steps", "5", "--warmup", "2"))
    assert out["config"]["workload"] == "stream_1f1b" and out["value"] > 0 and out["us_per_micro_batch"] > 0


@pytest.mark.gpu
@pytest.mark.parametrize("flag", ["--tags", "--accumulate", "--unbatched"])
def test_variant_runs_check_what_they_time(flag):
    out = one_line(run_bench("--steps", "10", "--warmup", "2", "--repeats", "5", "--regions", "cold", "--no-cpu-baseline",
                             "--no-staged", flag))
    assert out["value"] > 0 and out["roofline"]["frac"] > 0
