"""bench.py end to end on the GPU (short runs): one JSON line with the agreed fields, for the fused default path,
the two-call path and a HIP-graph run of a small workload."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

REQUIRED = ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
            "vs_baseline", "dtype", "data", "config", "roofline", "gradient", "mean", "timing")


def run_bench(*flags):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *flags], capture_output=True, text=True,
                       timeout=600, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1, r.stdout[-2000:]
    return json.loads(lines[0])


def check_common(out, steps, warmup):
    for key in REQUIRED:
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == steps and out["warmup"] == warmup
    assert out["unit"] == "worker-iters/s" and out["higher_is_better"] is True and out["vs_baseline"] is None
    assert out["data"] == "synthetic" and "workload" in out["config"] and "model" not in out["config"]
    assert out["value"] == pytest.approx(out["config"]["n"] / (out["ms_per_step"] * 1e-3), rel=1e-6)
    roof = out["roofline"]
    assert roof["bound"] == "hbm" and roof["unit"] == "GB/s" and roof["peak"] == 8000.0
    assert roof["frac"] == pytest.approx(roof["achieved"] / roof["peak"])
    assert 0.0 < roof["frac"] < 1.0
    assert roof["achieved"] == pytest.approx(roof["algorithmic_bytes_per_launch"] / (roof["avg_launch_ms"] * 1e-3) / 1e9)
    per = sorted(out["timing"]["ms_per_step_of_each_repeat"])
    assert len(per) == out["timing"]["repeats"]
    if "launch" not in out["config"]:
        assert out["ms_per_step"] == pytest.approx(per[len(per) // 2])      # the median repeat is the one reported


def test_default_workload_fused_path_short_run():
    out = run_bench("--steps", "3", "--warmup", "1", "--repeats", "3", "--no-cpu-baseline", "--no-others")
    check_common(out, 3, 1)
    assert "others" not in out
    assert out["config"]["workload"] == "mlp3_ring64" and out["config"]["path"] == "dpsgd_step"
    assert out["dtype"] == "bf16"
    assert "mlp_fused_ring_rows_kernel" in out["roofline"]["kernel"]
    assert out["roofline"]["algorithmic_bytes_per_launch"] == pytest.approx(8.0 * 64 * (3072 * 4096 + 4096 * 4096) / 2)
    # the counter figure comes from the committed summary of this workload, kernel and row stride
    assert out["roofline"]["traffic_source"].startswith("profiles/")
    assert out["roofline"]["traffic"] >= out["roofline"]["algorithmic_bytes_per_launch"]
    assert out["roofline"]["traffic"] < 1.2 * out["roofline"]["algorithmic_bytes_per_launch"]


def test_counter_traffic_is_reported_only_for_the_run_the_profile_describes():
    out = run_bench("--steps", "2", "--warmup", "1", "--repeats", "1", "--no-cpu-baseline", "--ld-multiple", "64")
    assert out["config"]["ld"] == 29409344                       # not the stride the profile was taken with
    assert out["roofline"]["traffic"] is None and out["roofline"]["traffic_source"] is None


def test_default_run_witnesses_every_workload():
    out = run_bench("--steps", "3", "--warmup", "1", "--repeats", "2", "--no-cpu-baseline")
    check_common(out, 3, 1)
    got = {(o["workload"], o["path"]) for o in out["others"]}
    assert got == {("mlp3_ring64", "dpsgd_grad + dpsgd_mix_step"), ("mlp3_torus8x8", "dpsgd_step"),
                   ("mlp3_torus8x8", "dpsgd_grad + dpsgd_mix_step"), ("mlp2_ring32", "dpsgd_step"),
                   ("resnet20_ring112", "dpsgd_grad + dpsgd_mix_step"), ("softmax_ring16", "dpsgd_grad + dpsgd_mix_step"),
                   ("lsq_ring8", "dpsgd_grad + dpsgd_mix_step")}
    for o in out["others"]:
        assert o["ms_per_step"] > 0 and 0.0 < o["frac"] < 1.0 and o["dominant_kernel"]
        assert o["value"] == pytest.approx({"mlp3_ring64": 64, "mlp3_torus8x8": 64, "mlp2_ring32": 32, "resnet20_ring112": 112,
                                            "softmax_ring16": 16, "lsq_ring8": 8}[o["workload"]] / (o["ms_per_step"] * 1e-3))
    two_call = [o for o in out["others"] if o["workload"] == "mlp3_ring64"][0]
    assert "mix_ring_fat_kernel" in two_call["dominant_kernel"]
    assert two_call["algorithmic_bytes_per_launch"] == pytest.approx(12.0 * 64 * 29409290)


def test_two_call_path_and_cpu_baseline_on_a_small_workload():
    out = run_bench("--workload", "softmax_ring16", "--steps", "5", "--warmup", "2", "--two-call", "--repeats", "3")
    check_common(out, 5, 2)
    assert out["dtype"] == "f32" and out["config"]["path"] == "dpsgd_grad + dpsgd_mix_step"
    assert out["roofline"]["algorithmic_bytes_per_launch"] == pytest.approx(12.0 * 16 * 30730)
    base = out["cpu_baseline"]
    assert base["kind"] == "oracle" and base["unit"] == "worker-iters/s" and base["cores"] >= 1 and base["value"] > 0
    assert isinstance(base["sample"], str) and base["sample"]
    assert base["single_thread"]["cores"] == 1 and base["single_thread"]["value"] > 0


def test_graph_run_reports_both_timings():
    out = run_bench("--workload", "lsq_ring8", "--steps", "20", "--warmup", "2", "--graph", "--no-cpu-baseline", "--repeats", "2")
    check_common(out, 20, 2)
    assert "HIP graph" in out["config"]["launch"] and out["config"]["eager_ms_per_step"] > 0
