"""bench.py's command line and the shape of the one JSON line it prints."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def test_more_than_one_gpu_is_refused_with_a_message():
    run = subprocess.run([sys.executable, BENCH, "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert run.returncode != 0
    assert "ONE GPU" in run.stderr and run.stdout.strip() == ""


@pytest.mark.gpu
def test_json_line_has_the_agreed_fields():
    run = subprocess.run([sys.executable, BENCH, "--steps", "2", "--warmup", "1", "--batch", "262144", "--cpu-sample", "4096"],
                         capture_output=True, text=True, timeout=600)
    assert run.returncode == 0, run.stderr
    lines = [l for l in run.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, "exactly one line on stdout"
    j = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling", "vs_baseline",
                "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in j, key
    assert j["n_gpus"] == 1 and j["steps"] == 2 and j["warmup"] == 1 and j["higher_is_better"] is True
    assert j["unit"] == "evals/s/party" and j["dtype"] == "u32" and j["data"] == "synthetic" and j["vs_baseline"] is None
    assert "workload" in j["config"] and "model" not in j["config"]
    r = j["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in r, key
    assert r["bound"] == "lds" and abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9 and 0 < r["frac"] < 1
    c = j["cpu_baseline"]
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in c, key
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0
    assert j["value"] > 100 * c["value"]          # sanity: the GPU path is not the oracle in disguise
