"""Host-side checks of bench.py that need no GPU: the one-GPU contract and the FLOP / byte accounting."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
from paper_1705_09056_amd import synth  # noqa: E402
from paper_1705_09056_amd.configs import by_name  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""


@pytest.mark.parametrize("name,flop", [
    ("lsq_ring8", 8 * 2 * 2 * 32 * 64),                                             # 65.5 K
    ("softmax_ring16", 16 * 4 * 128 * 3072 * 10),                                   # ~252 M
    ("mlp2_ring32", 32 * (4 * 128 * 3145728 + 6 * 128 * 10240)),                    # ~51.8 G
    ("mlp3_ring64", 64 * (4 * 32 * 12582912 + 6 * 32 * 16777216 + 6 * 32 * 40960)),  # ~310 G
])
def test_gradient_flop_counts_are_the_benchmark_definition(name, flop):
    """2MKN per GEMM; forward + weight gradient for a first layer, + data gradient for the others."""
    cfg = by_name(name)
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    g = bench.gradient_roofline(cfg, d, 1.0)
    assert g["flop_per_step"] == pytest.approx(flop, rel=1e-12)
    assert 0.0 < g["intensity_ceiling_frac"] <= 1.0
    assert g["frac_of_ceiling"] == pytest.approx(g["frac_of_peak"] / g["intensity_ceiling_frac"])


def test_cnn_flop_count_is_about_three_forward_passes():
    cfg = by_name("resnet20_ring112")
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    g = bench.gradient_roofline(cfg, d, 1.0)
    fwd_mac_per_image = 40.6e6            # stem 0.44 M + 6 x 2.36 M + (1.18 M + 5 x 2.36 M) x 2
    assert g["flop_per_step"] == pytest.approx(2 * 3 * fwd_mac_per_image * 32 * 112, rel=0.02)


def test_every_traffic_line_under_profiles_names_a_kernel_and_a_stride_that_exist():
    """The `bench-traffic:` lines bench.py reads its counter traffic from: each parses, names a kernel that is still in
    the sources, a benchmark workload, and the row stride bench.py gives that workload by default - a profile that has
    gone stale (a renamed kernel, a changed stride) fails here instead of silently yielding `traffic: null`."""
    import glob
    import json
    import re
    src = ""
    for f in glob.glob(os.path.join(ROOT, "paper_1705_09056_amd", "csrc", "*.hip")):
        with open(f) as fh:
            src += fh.read()
    lines = []
    for f in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        with open(f) as fh:
            lines += [(os.path.basename(f), ln) for ln in fh if "bench-traffic:" in ln]
    assert len(lines) >= 4
    for name, ln in lines:
        rec = json.loads(ln.split("bench-traffic:", 1)[1].strip())
        assert re.search(r"\b" + re.escape(rec["kernel"]) + r"\b", src), (name, rec["kernel"])
        cfg = by_name(rec["workload"])
        d = synth.model_dim(cfg.model_kind, cfg.widths)
        assert rec["ld"] >= d and rec["ld"] % 64 == 0
        assert rec["path"] in ("fused", "two-call")
        # the counted bytes are at least the algorithmic ones of that path and within 20 % of them
        n = cfg.n
        if rec["path"] == "two-call":
            assert 12.0 * n * d <= rec["bytes_per_launch"] <= 1.2 * 12.0 * n * d
        got, where = bench.traffic_from_profile(rec["workload"], rec["path"], rec["kernel"] + " (anything)", rec["ld"])
        assert got == rec["bytes_per_launch"] and where == name
