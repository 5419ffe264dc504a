"""bench.py's contract: one JSON line with the agreed fields; more than one GPU is refused."""
import json
import subprocess
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent


def run_bench(*flags, timeout=300):
    return subprocess.run([sys.executable, str(ROOT / "bench.py"), *flags], cwd=ROOT, capture_output=True, text=True, timeout=timeout)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run_bench("--gpus", "2")
    assert r.returncode != 0 and r.stdout.strip() == ""
    assert "ONE GPU" in r.stderr


def one_line(r):
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, r.stdout[-2000:]
    return json.loads(lines[0])


@pytest.mark.gpu
def test_the_bench_line_on_the_small_configuration(amlib):
    """The oracle finishes the 1M-parameter configuration in seconds, so the CPU leg and its parity gate run too."""
    d = one_line(run_bench("--workload", "tiny", "--steps", "7", "--warmup", "3"))
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "source_hash"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 7 and d["unit"] == "params/s" and d["vs_baseline"] is None
    assert d["config"]["name"] == "tiny" and "workload" in d["config"] and "model" not in d["config"]
    assert d["ms_per_step_segments"]["repeats"] == 5 and sum(d["ms_per_step_segments"]["steps_per_segment"]) == 7
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s" and r["launches"] == 7
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-12
    assert abs(r["achieved"] - r["algorithmic_bytes_per_launch"] / (r["kernel_ms"] * 1e-3) / 1e9) < 1e-6 * r["achieved"]
    assert r["kernel_ms_min"] <= d["ms_per_step_segments"]["max"]   # a kernel launch lies inside its step
    assert abs(d["value"] - d["config"]["replicas"] * d["config"]["n"] / (d["ms_per_step"] * 1e-3)) < 1e-6 * d["value"]
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0 and c["unit"] == "params/s"
    assert c["parity"]["max_rel_err_fp32"] < c["parity"]["tol_fp32"] == 1e-6


@pytest.mark.gpu
def test_the_bench_line_of_the_averaging_only_call(amlib):
    d = one_line(run_bench("--workload", "tiny", "--steps", "6", "--warmup", "3", "--averaging-only"))
    assert d["config"]["entry"] == "am_sparse_average" and "cpu_baseline" not in d
    r = d["roofline"]
    assert r["launches"] == 6 and r["traffic"] is None and r["kernel"].startswith("k_average")
    n, R, p = d["config"]["n"], d["config"]["replicas"], d["config"]["fraction"]
    assert abs(r["algorithmic_bytes_per_launch"] - 24.0 * p * R * n) < 1e-6 * r["algorithmic_bytes_per_launch"]
    assert r["line_granular_bytes_per_launch"] > r["algorithmic_bytes_per_launch"]
