"""bench.py keeps its output contract: one JSON line with the agreed keys, on the smallest workload."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu


def test_bench_prints_one_json_line_with_roofline_and_cpu_baseline(repo_root):
    res = subprocess.run([sys.executable, os.path.join(repo_root, "bench.py"), "--config", "0", "--steps", "5", "--warmup", "2"],
                         stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=300, cwd=repo_root)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, res.stdout
    j = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in j, key
    assert j["n_gpus"] == 1 and j["steps"] == 5 and j["warmup"] == 2 and j["higher_is_better"] is True
    assert j["value"] > 0 and j["ms_per_step"] > 0 and j["dtype"] == "f32" and j["data"] == "synthetic"
    assert "workload" in j["config"] and "model" not in j["config"]
    r = j["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in r, key
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3
    c = j["cpu_baseline"]
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in c, key
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0


def test_bench_refuses_more_than_one_gpu(repo_root):
    res = subprocess.run([sys.executable, os.path.join(repo_root, "bench.py"), "--gpus", "2"],
                         stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=120, cwd=repo_root)
    assert res.returncode != 0 and "ONE GPU" in res.stderr


def _bench_json(repo_root, *args):
    res = subprocess.run([sys.executable, os.path.join(repo_root, "bench.py"), *args],
                         stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=300, cwd=repo_root)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, res.stdout
    return json.loads(lines[0])


def test_epoch_ablation_mode_on_a_shrunk_graph(repo_root):
    """Section 3.3's claim at kernel level: the mode runs, only the transposition differs between its legs, and
    rebuilding the transpose every epoch costs more than looking it up."""
    j = _bench_json(repo_root, "--config", "1", "--shrink", "4", "--epoch-ablation", "4")
    for key in ("epoch_ms_cached_transpose", "epoch_ms_transpose_rebuilt", "transpose_ms", "backward_spmm_ms",
                "transpose_cost_in_backward_spmms", "speedup_from_cache", "first_epoch_ms_with_cache"):
        assert key in j and j[key] > 0, key
    assert j["epochs"] == 4 and j["epoch_ms_transpose_rebuilt"] > j["epoch_ms_cached_transpose"]


def test_width_sweep_mode_on_a_shrunk_graph(repo_root):
    """The GPU counterpart of the tuning graph (Section 3.2): every width of the sweep runs, including d = 8
    and widths that are not multiples of 4."""
    j = _bench_json(repo_root, "--config", "1", "--shrink", "4", "--sweep-d")
    widths = [p["d"] for p in j["sweep"]]
    assert widths == [8, 16, 30, 32, 64, 100, 128, 256, 512, 1024]
    assert all(p["ms"] > 0 and p["gflops"] > 0 and p["requested_GBps"] > 0 for p in j["sweep"])


def test_traffic_comes_from_the_tracked_counter_records(repo_root):
    """roofline.traffic is read from profiles/counter_records.txt (no byte constant in bench.py) and says which
    commit it was measured on."""
    sys.path.insert(0, repo_root)
    import bench
    rec = bench.counter_record("c3-rmat2.4m-d128", "k_spmm_grouped")
    assert rec and rec["bytes"] > 0 and rec["commit"]
    assert "35.42e9" not in open(os.path.join(repo_root, "bench.py")).read()


def test_split_rows_mode_on_a_shrunk_graph(repo_root):
    """Where a launch spends its time: the two row classes as matrices of their own cover every row and entry."""
    j = _bench_json(repo_root, "--config", "1", "--shrink", "4", "--split-rows", "64")
    a, b = j["classes"]
    assert a["class"] == "rows <= 64" and b["class"] == "rows > 64"
    assert a["rows"] > 0 and b["rows"] > 0 and a["ms"] > 0 and b["ms"] > 0
    import graphgen
    w = graphgen.make_config(1, shrink=4)
    assert a["rows"] + b["rows"] == w.n and a["entries"] + b["entries"] == w.nnz
