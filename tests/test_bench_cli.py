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


def test_all_cores_oracle_leg_computes_what_the_plain_calls_compute():
    """The threaded leg of bench.py's cpu_baseline only splits the edge list at destination boundaries and
    calls the unchanged oracle on each part: aggregates match bit for bit, the summed backward to rounding."""
    import numpy as np
    import oracle
    import bench
    from gen import workloads
    p = workloads.config3("f32", scale=0.01, upstream=False)
    rels = bench.layer_problem_relations(p, ("cites", "rev_writes"))
    for name, src, dst, n_s, n_t, table, W in rels:
        G = np.random.default_rng(1).standard_normal((n_t, W.shape[1])).astype(np.float32)
        M1, B1 = bench._oracle_relation(oracle, np, src, dst, n_s, n_t, table, W, G, "mean", 1)
        M4, B4 = bench._oracle_relation(oracle, np, src, dst, n_s, n_t, table, W, G, "mean", 4)
        assert np.array_equal(M1, M4), name
        assert np.allclose(B1, B4, rtol=1e-12, atol=1e-12), name
    rec = bench.cpu_baseline_both(rels, "mean", budget_s=0.2)
    assert rec["kind"] == "oracle" and rec["cores"] >= 1 and rec["single_thread"]["cores"] == 1 and rec["value"] > 0
