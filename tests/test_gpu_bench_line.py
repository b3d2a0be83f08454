"""The one JSON line bench.py prints, on the GPU, with a short run of the headline workload: the keys of the contract,
the roofline object's arithmetic, and the CPU-oracle baseline beside it."""

import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_the_headline_line_has_the_contracts_keys_and_consistent_figures():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "6", "--warmup", "2", "--reps", "1", "--cpu-steps", "2"],
                       capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [l for l in p.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1, p.stdout[-2000:]
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling", "vs_baseline",
              "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 6 and d["warmup"] == 2 and d["unit"] == "GB/s" and d["data"] == "synthetic"
    assert d["vs_baseline"] is None and d["higher_is_better"] is True and "workload" in d["config"] and "model" not in d["config"]
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s" and r["kernel"] == "mw_k_copy"
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3
    # achieved = algorithmic bytes per launch / average launch duration; the step cannot be shorter than its kernel
    assert abs(r["achieved"] - r["alg_bytes_per_launch"] / (r["avg_launch_ms"] * 1e-3) / 1e9) < 0.01 * r["achieved"]
    assert r["avg_launch_ms"] <= d["ms_per_step"] * 1.02 and 0.5 < r["frac"] < 1.0
    # payload rate = payload bytes per step / step time
    assert abs(d["value"] - d["config"]["payload_bytes_per_step"] / (d["ms_per_step"] * 1e-3) / 1e9) < 0.01 * d["value"]
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] == 1 and c["unit"] == "GB/s" and 0 < c["value"] < d["value"] and c["sample"]


OTHER_WORKLOADS = [
    ["--workload", "config1", "--reps", "1"],
    ["--workload", "config3", "--steps", "100", "--reps", "1"],
    ["--workload", "config4", "--steps", "30", "--abort-step", "10", "--reps", "1"],
    ["--workload", "config5", "--ops", "600", "--reps", "0"],
    ["--workload", "collectives", "--coll-launches", "3", "--coll-warmup", "1"],
    ["--workload", "sweep", "--reps", "1"],
    ["--workload", "online", "--reps", "1"],
]


@pytest.mark.parametrize("args", OTHER_WORKLOADS, ids=[a[1] for a in OTHER_WORKLOADS])
def test_every_other_workloads_line_carries_roofline_and_cpu_baseline(args):
    """Short runs of the other --workload lines: one JSON line each, with the contract's keys, a roofline object for the
    dominant kernel (bound, achieved, peak, frac consistent) and the CPU oracle's baseline on a stated sample."""
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [l for l in p.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1, p.stdout[-2000:]
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling", "vs_baseline",
              "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["value"] > 0 and d["vs_baseline"] is None and "workload" in d["config"]
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s" and r["kernel"].startswith("mw_k_")
    assert 0 < r["achieved"] < r["peak"] and abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] == 1 and c["value"] > 0 and c["sample"]
