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


def test_traffic_table_names_every_workload_and_its_commit():
    """bench.py reads roofline.traffic from the tracked profiler summary: every workload must be
    there with plausible bytes, and the table must say which commit it was measured at."""
    sys.path.insert(0, ROOT)
    import bench
    table, commit = bench.traffic_table()
    assert commit and len(commit) >= 7
    assert set(table) == set(bench.WORKLOADS)
    for name, row in table.items():
        assert row["gemm"] > 1e8 and row["quant"] > 5e7, name
    # quantization traffic equals its algorithmic bytes (read 2 B, write 1 B per element + scales)
    assert abs(table["qkv256"]["quant"] / (16384 * 1152 * 3 + 4 * 16384) - 1) < 0.02
    assert abs(table["fc2_512_w8"]["quant"] / (65536 * 4608 * 3 + 4 * 65536) - 1) < 0.02
    # the GEMM never moves less than its algorithmic bytes
    assert table["fc1_512"]["gemm"] > 65536 * 1152 + 4608 * 1152 + 65536 * 4608 * 2


def test_roofs_program_is_built_beside_the_library():
    assert os.path.exists(os.path.join(ROOT, "bench", "qc_roofs.hip"))
    assert os.access(os.path.join(ROOT, "bench", "qc_roofs"), os.X_OK), "run python -m paper_2503_06545_amd.build"


CONTRACT_KEYS = ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step",
                 "higher_is_better", "scaling", "vs_baseline", "dtype", "data", "config",
                 "roofline", "cpu_baseline")


def run_bench(extra):
    r = subprocess.run([sys.executable, BENCH] + extra, capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in CONTRACT_KEYS:
        assert key in d, key
    assert d["n_gpus"] == 1 and d["data"] == "synthetic"
    assert d["vs_baseline"] is None and d["higher_is_better"] is True
    assert "workload" in d["config"] and "model" not in d["config"]
    return d


def check_roofline(rf):
    assert rf["bound"] == "mfma" and rf["unit"] == "TOP/s" and rf["peak"] == 5000.0
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3 and 0.05 < rf["frac"] < 1.0
    ach = rf["achievable"]
    assert 1000 < ach["mfma_with_the_gemms_operand_traffic"] < ach["mfma_registers_only_random_operands"] <= 5100
    assert abs(rf["frac_of_achievable"] - rf["achieved"] / ach["mfma_registers_only_random_operands"]) < 1e-3


@pytest.mark.gpu
def test_default_run_is_the_sweep_with_the_single_layer_configurations():
    """The command the round's end runs (with fewer steps): headline = the 28-block sweep."""
    d = run_bench(["--gpus", "1", "--steps", "3", "--warmup", "1"])
    assert d["steps"] == 3 and d["warmup"] == 1
    assert d["config"]["name"] == "sweep28" and "M = 131072" in d["config"]["workload"]
    assert d["config"]["layers"] == 112 and 20 <= d["config"]["w4_layers"] <= 50
    ops = sum(2.0 * 131072 * n * k for n, k in ((3456, 1152), (1152, 1152), (4608, 1152), (1152, 4608))) * 28
    assert abs(d["value"] - ops / (d["ms_per_step"] * 1e-3) / 1e12) < 0.01 * d["value"]
    check_roofline(d["roofline"])
    assert d["roofline"]["launches_per_step"] == 112
    assert d["device"]["samples"] > 10           # the timed region is long enough to sample
    roofs = d["achievable_roofs"]
    assert 3000 < roofs["hbm_read_gbs"] < 8000 and 3000 < roofs["hbm_copy_gbs"] < 8000
    assert 3000 < roofs["hbm_read2_write1_gbs"] < 8000
    assert d["kernels"]["quant_act"]["achievable"] == roofs["hbm_read2_write1_gbs"]
    assert roofs["read_32mib_cold_us"] > roofs["read_32mib_warm_us"] > 1.0
    assert len(d["provenance"]["source_sha16"]) == 16 and d["provenance"]["rocm"]
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] >= 1 and cb["value"] > 0 and cb["sample"]
    assert d["value"] > 100 * cb["value"] and len(cb["classes"]) == 8
    k = d["kernels"]
    assert k["qlinear_whole_call"]["achieved"] < d["roofline"]["achieved"]
    assert {c["layer"] for c in k["gemm_by_layer_class"]} == {"qkv", "out", "fc1", "fc2"}
    assert set(d["configs"]) == {"qkv256", "fc1_512", "fc2_512_w8", "fc2_512_w4"}
    for name, c in d["configs"].items():
        check_roofline(c["roofline"])
        assert abs(c["value"] - 2.0 * c["M"] * c["N"] * c["K"] / (c["ms_per_step"] * 1e-3) / 1e12) < 0.01 * c["value"]
        assert c["kernels"]["quant_act"]["frac"] > 0.2 and c["kernels"]["latent_delta"]["avg_launch_us"] > 0
        assert c["kernels"]["qlinear_whole_call"]["achieved"] < c["roofline"]["achieved"]
        assert c["device"]["samples"] > 10
    for name in ("qkv256", "fc1_512"):
        k = d["configs"][name]["kernels"]
        assert k["quant_act"]["cold"]["avg_launch_us"] > 0 and k["latent_delta"]["cold"]["avg_launch_us"] > 0
        assert 0.3 < k["latent_delta"]["cold"]["frac_of_read_only_kernel"] <= 1.05


@pytest.mark.gpu
def test_single_layer_headline_with_another_activation_quantizer():
    d = run_bench(["--workload", "qkv256", "--variant", "asym", "--steps", "20", "--warmup", "20",
                   "--library-gemm"])
    assert d["steps"] == 20 and d["warmup"] == 20 and "configs" not in d
    lib = d["library_int8_gemm"]["shapes"]
    assert set(lib) == {"16384x1152x3456"}
    assert all("error" in v or 0 < v["frac"] < 1 for v in lib.values())
    assert 0 < d["library_int8_gemm"]["square_8192"]["qc_qlinear_gemm"]["frac"] < 1
    check_roofline(d["roofline"])
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] >= 1 and cb["value"] > 0 and cb["sample"]
    assert d["value"] > 100 * cb["value"] and 0 < cb["one_thread"]["value"] <= cb["value"]
    k = d["kernels"]
    assert k["quant_act"]["cold"]["avg_launch_us"] > 0 and k["latent_delta"]["cold"]["avg_launch_us"] > 0
    assert k["qlinear_whole_call"]["achieved"] < d["roofline"]["achieved"]
    assert abs(d["value"] - 2.0 * 16384 * 3456 * 1152 / (d["ms_per_step"] * 1e-3) / 1e12) < 0.01 * d["value"]
