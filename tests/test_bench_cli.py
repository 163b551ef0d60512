"""Host-side checks of the benchmark's command line and of the profiler-summary tool (no GPU)."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, cwd=ROOT)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)


def test_traffic_files_name_the_kernels_the_benchmark_reports():
    """profiles/traffic_*.json (written by the profiler-summary tool, read by bench.py for roofline.traffic)
    hold per-launch HBM bytes under the library's kernel names."""
    for name in ("traffic_config3_f32.json", "traffic_config3_bf16.json", "traffic_config4_bf16.json"):
        with open(os.path.join(ROOT, "profiles", name)) as f:
            rec = json.load(f)
        assert any(k.startswith("agg_") for k in rec) and any(k.startswith("gemm_") for k in rec)
        for k, v in rec.items():
            assert v["hbm_bytes_per_launch"] >= 0 and v["launches"] > 0, k
