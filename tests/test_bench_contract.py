"""The benchmark's command-line contract: one GPU only, one JSON line with the agreed keys."""
import json
import os
import subprocess
import sys

import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, BENCH, "--gpus", "2"], capture_output=True, text=True, cwd=ROOT, timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr
    assert res.stdout.strip() == ""


def test_stored_counter_traffic_is_only_used_for_the_rank_it_was_measured_at():
    sys.path.insert(0, ROOT)
    import bench
    name = "gemm_products_cfg2_vitb_fc1_hbm_traffic.txt"
    assert bench.read_traffic(name, 8, "l1") > 1e7
    assert bench.read_traffic(name, 36, "l1") is None
    assert bench.read_traffic(name, 8, "linf") is None
    assert bench.read_traffic("no_such_profile.txt", 8, "l1") is None


@pytest.mark.gpu
def test_one_json_line_with_the_agreed_keys():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    res = subprocess.run([sys.executable, BENCH, "--steps", "20", "--warmup", "5"], capture_output=True, text=True,
                         cwd=ROOT, timeout=600)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    j = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in j, key
    assert j["n_gpus"] == 1 and j["steps"] == 20 and j["warmup"] == 5
    assert j["vs_baseline"] is None and j["data"] == "synthetic" and j["dtype"] == "bf16"
    assert j["config"]["workload"] == "cfg2_vitb_fc1" and "model" not in j["config"]
    assert j["value"] > 0 and j["ms_per_step"] > 0
    roof = j["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in roof, key
    assert roof["bound"] in ("hbm", "mfma", "alu")
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3
    # measurement protocol: medians over at least 100 launches whatever --steps says, so the parts
    # of a call cannot exceed the whole
    st = j["stages"]
    assert st["projection_us"] + st["products_us"] <= 1.1 * j["ms_per_step"] * 1e3, (st, j["ms_per_step"])
    assert roof["launches"] >= 100 and abs(roof["avg_launch_us"] - roof["mean_launch_us"]) <= 0.1 * roof["avg_launch_us"]
    # the table of every configuration, rank and order
    rows = {(r["workload"], r["r"], r["order"]) for r in j["sweep"]}
    sys.path.insert(0, ROOT)
    import bench
    from paper_2309_15275_amd import workloads
    assert rows == set(bench.sweep_cases(workloads)) and len(rows) == 25
    for row in j["sweep"]:
        assert row["lbp_us"] > 0 and row["full_bp_us"] > 0 and abs(row["speedup"] - row["full_bp_us"] / row["lbp_us"]) < 0.02
        assert 0 < row["proj_frac_hbm"] < 1
    cpu = j["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["value"] > 0 and cpu["cores"] >= 1 and cpu["sample"]
