"""bench.py's command-line contract: what it refuses without a GPU (CPU test), and the shape of
the one JSON line it prints on the GPU (reduced launch counts; the figures are not asserted)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def run(*args, timeout=600):
    return subprocess.run([sys.executable, BENCH, *args], capture_output=True, text=True, timeout=timeout, cwd=ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    p = run("--gpus", "2", timeout=120)
    assert p.returncode != 0
    assert "one GPU" in p.stderr and p.stdout.strip() == ""


def test_unknown_section_is_refused():
    p = run("--sections", "step,nonsense", timeout=120)
    assert p.returncode != 0 and "unknown section" in p.stderr


@pytest.mark.gpu
def test_json_line_has_the_contract_fields():
    p = run("--sections", "step,c3", "--steps", "3", "--warmup", "1", "--launches", "5", "--reps", "1")
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [l for l in p.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, "exactly one line on stdout"
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "kernels"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["unit"] == "GB/s"
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and "workload" in d["config"]
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3
    assert r["traffic"] > 0 and "traffic_source" in r
    # the dominant kernel's figure follows from the algorithmic bytes and the measured duration
    assert abs(r["achieved"] - r["algo_bytes_per_launch"] / r["avg_launch_us"] / 1e3) < 1.0
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0 and c["sample"]
    assert d["rows_checked_against_oracle"] >= 5
    assert d["rows_matching_oracle"] == d["rows_checked_against_oracle"]
    assert 0 < d["value"] <= 8000.0 and abs(d["value"] - d["config"]["algo_bytes_per_step"] / d["ms_per_step"] / 1e6) < 2.0
