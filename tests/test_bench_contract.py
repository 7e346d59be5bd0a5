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
    assert r["bound"] == "lds" and abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-4 and 0 < r["frac"] < 1
    c = j["cpu_baseline"]
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in c, key
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0
    assert j["value"] > 100 * c["value"]          # sanity: the GPU path is not the oracle in disguise


@pytest.mark.gpu
def test_default_line_carries_both_rooflines_every_configuration_and_the_clock():
    """The default command (shortened: fewer steps and repetitions, a smaller oracle sample) on the
    2^22 configuration: KeyGen roofline beside the Eval one, the sustained clock, the oracle baseline
    with its parity statement, and one entry per benchmark configuration."""
    run = subprocess.run([sys.executable, BENCH, "--steps", "2", "--warmup", "1", "--config-reps", "3", "--cpu-sample", "16384"],
                         capture_output=True, text=True, timeout=900)
    assert run.returncode == 0, run.stderr
    lines = [l for l in run.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    j = json.loads(lines[0])
    assert j["config"]["batch"] == 1 << 22 and "2^22" not in j["metric"] and j["metric"].startswith("FSS comparison evals/sec per party")
    r = j["roofline"]
    assert r["bound"] == "lds" and r["kernel"] == "eval_kernel<cmp>" and 0.5 < r["frac"] < 1.1
    assert r["frac_issued"] < r["frac"] and r["traffic"] is not None
    assert abs(r["traffic"] / r["traffic_algorithmic"] - 1) < 0.01
    g = r["gen"]
    assert g["kernel"] == "gen_kernel<cmp>" and 0.5 < g["frac"] < 1.2 and g["frac_issued"] < g["frac"]
    assert 1000 < j["sustained_clock_mhz"] < 2600 and j["nominal_clock_mhz"] == 2400
    assert "parity" in j["cpu_baseline"] and "same alpha" in j["cpu_baseline"]["sample"]
    names = [c["name"] for c in j["configs"]]
    assert names == ["config1", "config2", "config3", "config4", "config5", "n16"]
    for c in j["configs"]:
        for key in ("eval_ms", "gen_ms", "evals_per_s", "pairs_per_s", "kernel", "warmup_steps"):
            assert key in c, (c["name"], key)
        assert c["eval_ms"][1] <= c["eval_ms"][0] and c["gen_ms"][1] <= c["gen_ms"][0]          # [median, min]
        for lds, issued, alu, hbm in (c["eval_frac"], c["gen_frac"]):
            assert 0 < issued <= lds * 1.02 and 0 < hbm < 1 and 0 < alu < 1
    assert "median" in j["configs_legend"]
    assert len(lines[0]) < 4000, "the line must stay short enough to survive a log tail"
    assert j["configs"][0]["kernel"] == "eval_octo_kernel<cmp>" and j["configs"][1]["kind"] == "eq" and j["configs"][3]["rounds"] == 8
