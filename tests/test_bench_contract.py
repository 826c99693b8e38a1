"""Host-side checks of the measurement contract: bench.py refuses more than one GPU with a message, and the bench
line stored with the profiles carries every field the contract names."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert p.returncode == 2
    assert "ONE GPU" in p.stderr and p.stdout.strip() == ""


def test_stored_bench_line_has_the_contract_fields():
    line = json.load(open(os.path.join(ROOT, "profiles", "production_bench_line.json")))
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in line, key
    assert line["n_gpus"] == 1 and line["vs_baseline"] is None and line["data"] == "synthetic"
    assert line["config"]["workload"] == "production" and "model" not in line["config"]
    r = line["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in r, key
    assert r["bound"] == "mfma" and r["unit"] == "TFLOP/s" and abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9
    c = line["cpu_baseline"]
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in c, key
    assert c["kind"] == "oracle"
    # value is whole-job throughput of the timed steps
    n_scores = line["config"]["sum_M"]
    assert abs(line["value"] - n_scores / (line["ms_per_step"] * 1e-3)) / line["value"] < 1e-6
