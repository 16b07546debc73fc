"""bench.py prints one JSON line with the agreed fields (run on the small `tiny` workload)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, timeout=600)
    return r


def test_bench_line_has_the_contract_fields():
    r = _run("--workload", "tiny", "--steps", "4", "--warmup", "2")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 4 and d["warmup"] == 2 and d["higher_is_better"] is True
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and d["config"]["workload"] == "tiny"
    assert d["value"] > 0 and abs(d["ms_per_step"] * d["value"] - 1000.0) < 1e-6 * 1000.0
    t = d["timing"]
    assert t["reps"] >= 5 and t["min_ms"] <= t["median_ms"] <= t["max_ms"]
    assert abs(t["median_ms"] - d["ms_per_step"] * d["steps"]) < 1e-6 * t["median_ms"]
    assert d["full_epoch"]["batches"] == 4 and d["full_epoch"]["batches_per_s_median"] > 0
    assert d["config"]["GPU_MAX_HW_QUEUES"] is not None
    roof = d["roofline"]
    assert roof["bound"] == "hbm" and roof["unit"] == "GB/s" and roof["peak"] == 8000.0
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-12
    assert roof["traffic"] is None and roof["traffic_source"] is None        # no counter run is recorded for `tiny`
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] == 1 and cpu["value"] > 0 and cpu["unit"] == d["unit"]
    g = d["gather"]
    assert g["rows"] == g["n_local"] + g["n_hit"] + g["n_miss"]
    pts = d["cache_hit_curve"]["points"]
    assert [p["hit_pct"] for p in pts] == sorted(p["hit_pct"] for p in pts) and abs(pts[-1]["hit_pct"] - 100.0) < 1e-9


def test_bench_refuses_more_than_one_gpu():
    r = _run("--gpus", "2")
    assert r.returncode != 0 and "one GPU" in r.stderr
