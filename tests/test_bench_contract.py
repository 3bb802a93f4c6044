"""The benchmark's command-line contract: one JSON line with the agreed fields; more than one GPU
is refused with a message (this library has no multi-GPU path)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       cwd=ROOT, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.gpu
@pytest.mark.parametrize("extra,workload", [
    # the default run: the update minibatch (the largest single-GPU configuration), forward + backward
    (["--steps", "3", "--warmup", "1", "--cpu-baseline-states", "1"], "config 5"),
    (["--config", "2", "--steps", "5", "--warmup", "2", "--cpu-baseline-seconds", "2"], "config 2")])
def test_bench_prints_one_json_line_with_roofline_and_cpu_baseline(extra, workload):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")] + extra, capture_output=True, text=True,
                       cwd=ROOT, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert d["config"]["workload"].startswith(workload)
    assert ("backward" in d["config"]["workload"]) == (workload == "config 5")
    assert "segment_sum" in d and d["segment_sum"]["bound"] == "hbm" and 0 < d["segment_sum"]["frac"] < 1
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == int(extra[extra.index("--steps") + 1]) and d["vs_baseline"] is None
    assert d["unit"] == "graphs/s" and d["value"] > 0 and d["data"] == "synthetic" and "workload" in d["config"]
    assert abs(d["value"] - d["config"]["graphs"] / (d["ms_per_step"] * 1e-3)) <= 1e-6 * d["value"]
    rf = d["roofline"]
    for k in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert k in rf, k
    assert rf["bound"] in ("hbm", "mfma", "alu") and rf["peak"] > 0
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) <= 1e-9 and 0 < rf["frac"] < 1
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["value"] > 0 and cb["cores"] >= 1 and cb["unit"] == "graphs/s" and cb["sample"]
