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
            "vs_baseline", "dtype", "data", "config", "roofline", "gradient", "mean")


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


def test_default_workload_fused_path_short_run():
    out = run_bench("--steps", "3", "--warmup", "1", "--no-cpu-baseline")
    check_common(out, 3, 1)
    assert out["config"]["workload"] == "mlp3_ring64" and out["config"]["path"] == "dpsgd_step"
    assert out["dtype"] == "bf16"
    assert "mlp_fused_ring_rows_kernel" in out["roofline"]["kernel"]
    assert out["roofline"]["algorithmic_bytes_per_launch"] == pytest.approx(8.0 * 64 * (3072 * 4096 + 4096 * 4096) / 2)
    assert out["roofline"]["traffic"] is not None and out["roofline"]["traffic"] >= out["roofline"]["algorithmic_bytes_per_launch"]


def test_two_call_path_and_cpu_baseline_on_a_small_workload():
    out = run_bench("--workload", "softmax_ring16", "--steps", "5", "--warmup", "2", "--two-call")
    check_common(out, 5, 2)
    assert out["dtype"] == "f32" and out["config"]["path"] == "dpsgd_grad + dpsgd_mix_step"
    assert out["roofline"]["algorithmic_bytes_per_launch"] == pytest.approx(12.0 * 16 * 30730)
    base = out["cpu_baseline"]
    assert base["kind"] == "oracle" and base["unit"] == "worker-iters/s" and base["cores"] >= 1 and base["value"] > 0
    assert isinstance(base["sample"], str) and base["sample"]


def test_graph_run_reports_both_timings():
    out = run_bench("--workload", "lsq_ring8", "--steps", "20", "--warmup", "2", "--graph", "--no-cpu-baseline")
    check_common(out, 20, 2)
    assert "HIP graph" in out["config"]["launch"] and out["config"]["eager_ms_per_step"] > 0
