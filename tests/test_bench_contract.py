"""bench.py's command-line contract: one GPU only, and one JSON line with the agreed keys."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, BENCH, "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout == ""


@pytest.mark.gpu
@pytest.mark.parametrize("extra", [[], ["--variant", "asym"]])
def test_one_json_line_with_the_contract_keys(extra):
    r = subprocess.run([sys.executable, BENCH, "--steps", "20", "--warmup", "20"] + extra,
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step",
                "higher_is_better", "scaling", "vs_baseline", "dtype", "data", "config",
                "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 20 and d["warmup"] == 20 and d["data"] == "synthetic"
    assert d["vs_baseline"] is None and d["higher_is_better"] is True
    assert "workload" in d["config"] and "model" not in d["config"]
    rf = d["roofline"]
    assert rf["bound"] == "mfma" and rf["unit"] == "TOP/s" and rf["peak"] == 5000.0
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3 and 0.05 < rf["frac"] < 1.0
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] >= 1 and cb["value"] > 0 and cb["sample"]
    assert d["value"] > 100 * cb["value"] and 0 < cb["one_thread"]["value"] <= cb["value"]
    k = d["kernels"]
    assert k["quant_act"]["cold"]["avg_launch_us"] > 0 and k["latent_delta"]["cold"]["avg_launch_us"] > 0
    assert k["qlinear_whole_call"]["achieved"] < rf["achieved"]
    assert abs(d["value"] - 2.0 * 16384 * 3456 * 1152 / (d["ms_per_step"] * 1e-3) / 1e12) < 0.01 * d["value"]
