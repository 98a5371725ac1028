#!/usr/bin/env python3
"""Benchmark of the quantized-linear hot path on one MI355X.

A step is one pass of the per-step hot path over one batch of seeded synthetic input.  The
default workload, and the headline of the JSON line, is the largest single-GPU configuration:
the 28-block STDiT linear sweep at M = 131072 tokens (CFG batch 2 at 512x512), 112 qc_qlinear
calls per step (per-token activation quantization + int8 MFMA GEMM + dequant/bias/GELU
epilogue) with the per-layer weight bit-width from the seeded importance mask.  The same run
then times the single-layer configurations (QKV 256x256, fc1 + GELU 512x512, fc2 512x512 with
int8 and with int4 weights, each with qc_latent_delta on a second stream) and reports them
under `configs`, each with its own GEMM-only and whole-call TOPS, quantization GB/s and
roofline.  `--workload NAME` makes one of those the headline instead (then without the
others); `--variant` selects how the activations are quantized.

Before the library touches the GPU, the stand-alone micro-benchmark bench/qc_roofs runs as a
child process and measures what this machine sustains (HBM streams, the int8 MFMA loop on random
operands with and without the GEMM's operand traffic); every roofline carries the fraction of
the nominal peak and of those measured roofs.  Before any timed region the GPU is loaded for a
fixed time, whatever --warmup says, so that the clocks have ramped up.

Weights are packed once before the timed region (an offline step of the method); inputs are
resident in HBM when timing starts.  Prints ONE JSON line.  `value` = integer ops (2*M*N*K per
layer) of the step divided by the step time.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0   # MI355X dense int8 MFMA, 5.0 POP/s
PEAK_HBM_GBS = 8000.0     # MI355X HBM3E, 8 TB/s
PRELOAD_SECONDS = 0.3     # load on the GPU before every timed region, independent of --warmup

SINGLE = ("qkv256", "fc1_512", "fc2_512_w8", "fc2_512_w4")
WORKLOADS = ("sweep28",) + SINGLE
# How the activations are quantized: the spec form (symmetric int8 per token), the lower
# activation bit-widths of Eq. (8), the rotation fused into the quantization, or the printed
# asymmetric form of Eq. (3)-(4).  The GEMM is the same kernel in all of them.
VARIANTS = {"a8": dict(act_bits=8), "a6": dict(act_bits=6), "a4": dict(act_bits=4),
            "rot128": dict(act_bits=8, rot=128), "asym": dict(act_bits=8, asym=True)}
VARIANT_TEXT = {"a8": "symmetric int8 per token", "a6": "symmetric 6 bit per token",
                "a4": "symmetric 4 bit per token",
                "rot128": "Walsh-Hadamard blocks of 128 columns, then symmetric int8 per token",
                "asym": "asymmetric uint8 per token with zero point"}
DESCRIBE = {
    "sweep28": "28 STDiT blocks x (QKV 1152->3456, out 1152->1152, fc1 1152->4608 + GELU, "
               "fc2 4608->1152), M = 131072 tokens (CFG batch 2 at 512x512), bf16 in/out, "
               "per-layer weight bit-width from the seeded mask (BASELINE configs[4])",
    "qkv256": "STDiT QKV projection 256x256 (BASELINE configs[1]): X bf16 [16384,1152] N(0,1) with "
              "12 outlier columns x20, W8A8 [3456,1152], bias, bf16 out; + latent delta on "
              "2 x [16,4,16,64,64] fp32",
    "fc1_512": "STDiT MLP fc1 + GELU(tanh) 512x512 (BASELINE configs[2]): X bf16 [65536,1152], "
               "W8A8 [4608,1152], bf16 out; + latent delta on 2 x [16,4,16,64,64] fp32",
    "fc2_512_w8": "STDiT MLP fc2 512x512 (BASELINE configs[3]): X bf16 [65536,4608] post-GELU, "
                  "W8A8 [1152,4608], bf16 out; + latent delta on 2 x [16,4,16,64,64] fp32",
    "fc2_512_w4": "STDiT MLP fc2 512x512 (BASELINE configs[3]): X bf16 [65536,4608] post-GELU, "
                  "W4A8 [1152,4608] int4 weights, bf16 out; + latent delta on 2 x [16,4,16,64,64] fp32",
}
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")


# ---- measured roofs, provenance ------------------------------------------------------------

def measured_roofs():
    """Run bench/qc_roofs --quick as a child process (it must finish before this process uses
    the GPU) and return its "@key value" lines."""
    exe = os.path.join(ROOT, "bench", "qc_roofs")
    if not os.path.exists(exe):
        return {"error": "bench/qc_roofs is not built (python -m paper_2503_06545_amd.build)"}
    t0 = time.perf_counter()
    try:
        r = subprocess.run([exe, "--quick"], capture_output=True, text=True, timeout=120)
    except subprocess.TimeoutExpired:
        return {"error": "bench/qc_roofs --quick did not finish in 120 s"}
    if r.returncode != 0:
        return {"error": f"bench/qc_roofs exited with {r.returncode}: {r.stdout[-300:]}"}
    out = {}
    for line in r.stdout.splitlines():
        if line.startswith("@"):
            k, v = line[1:].split()
            out[k] = float(v)
    out["seconds"] = round(time.perf_counter() - t0, 1)
    out["source"] = "bench/qc_roofs --quick, child process of this run, same GPU"
    return out


def traffic_table():
    """HBM-side bytes per launch from the tracked rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE passes scaled by a plain copy): {workload: {kernel: bytes}}, the commit it was
    measured at."""
    table, commit = {}, None
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                p = line.split()
                if len(p) >= 2 and p[0] == "measured_at_commit":
                    commit = p[1]
                elif len(p) == 4 and p[0] == "traffic":
                    table.setdefault(p[1], {})[p[2]] = float(p[3])
    except OSError:
        pass
    return table, commit


def provenance():
    import torch
    h = hashlib.sha256()
    files = ["bench.py", "include/qc.h"] + sorted(
        os.path.join("paper_2503_06545_amd", "csrc", f)
        for f in os.listdir(os.path.join(ROOT, "paper_2503_06545_amd", "csrc")))
    for f in files:
        with open(os.path.join(ROOT, f), "rb") as fh:
            h.update(fh.read())
    head = None
    try:
        r = subprocess.run(["git", "-C", ROOT, "describe", "--always", "--dirty", "--abbrev=12"],
                           capture_output=True, text=True, timeout=10)
        head = r.stdout.strip() or None
    except (OSError, subprocess.TimeoutExpired):
        pass
    if head is None:  # the GPU machine gets the tree without its history: take the build's stamp
        try:
            with open(os.path.join(ROOT, "paper_2503_06545_amd", "_build", "build_info.json")) as f:
                head = json.load(f).get("git") + " (at build time)"
        except (OSError, ValueError, TypeError):
            pass
    rocm = None
    try:
        with open("/opt/rocm/.info/version") as f:
            rocm = f.read().strip()
    except OSError:
        pass
    return {"git": head, "source_sha16": h.hexdigest()[:16],
            "source_sha16_of": "bench.py, include/qc.h, paper_2503_06545_amd/csrc/*",
            "rocm": rocm, "torch": torch.__version__, "hip": torch.version.hip}


# ---- timing helpers ---------------------------------------------------------------------------

def batch_times_us(fn, batch, rounds):
    """Average duration of one fn() from HIP events around batches of back-to-back calls
    (a batch keeps the GPU loaded and amortises the dispatch gap that an event pair around a
    single launch would include).  The events are recorded on torch's current stream, which is
    the stream every timed kernel is launched on."""
    import torch
    t = []
    for _ in range(rounds):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(batch):
            fn()
        e1.record()
        e1.synchronize()
        t.append(e0.elapsed_time(e1) * 1e3 / batch)
    return {"avg_us": sum(t) / len(t), "min_us": min(t)}


def preload(fn, seconds=PRELOAD_SECONDS):
    """Keep the GPU busy with fn() for a fixed time so that its clocks have ramped up."""
    import torch
    t0 = time.perf_counter()
    n = 0
    while time.perf_counter() - t0 < seconds:
        fn()
        n += 1
        if n % 8 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    return n


class PowerSampler:
    """Reads the GPU's socket power and shader clock from sysfs every few milliseconds while
    the timed loop runs (best effort: missing files give None)."""

    def __init__(self):
        import glob
        import threading
        self.power_file = (glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input") + [None])[0]
        self.cap_file = (glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_cap") + [None])[0]
        self.clk_file = (glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk") + [None])[0]
        self.power, self.clock = [], []
        self._stop = threading.Event()
        self._thread = threading.Thread(target=self._run, daemon=True)

    @staticmethod
    def _read(path):
        try:
            with open(path) as f:
                return f.read()
        except (OSError, TypeError):
            return None

    def _run(self):
        while not self._stop.is_set():
            p = self._read(self.power_file)
            if p:
                self.power.append(int(p) * 1e-6)
            c = self._read(self.clk_file)
            if c:
                for line in c.splitlines():
                    if "*" in line:
                        self.clock.append(float(line.split(":")[1].lower().replace("mhz", "").replace("*", "")))
            self._stop.wait(0.005)

    def __enter__(self):
        self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop.set()
        self._thread.join()

    def summary(self):
        cap = self._read(self.cap_file)
        avg = lambda v: round(sum(v) / len(v), 1) if v else None
        return {"power_cap_w": round(int(cap) * 1e-6, 1) if cap else None,
                "power_w_avg": avg(self.power), "power_w_max": round(max(self.power), 1) if self.power else None,
                "shader_clock_mhz_avg": avg(self.clock), "samples": len(self.power)}


# ---- CPU baseline: the oracle as it stands -----------------------------------------------------

def _oracle_linear(case, layer, act_bits, rot, asym):
    import oracle
    W, b = case.weight(layer), case.bias(layer)
    qw, sw = oracle.quant_weight_rot(W, case.bits, rot) if rot else oracle.quant_weight(W, case.bits)
    epi = {"none": oracle.EPI_NONE, "gelu_tanh": oracle.EPI_GELU_TANH,
           "gelu_erf": oracle.EPI_GELU_ERF}[case.epi]

    def linear(x):
        if asym:
            return oracle.qlinear_asym(x, qw, sw, b, epi, act_bits)
        if rot:
            return oracle.qlinear_rot(x, qw, sw, rot, b, epi, act_bits)
        return oracle.qlinear(x, qw, sw, b, epi, act_bits)
    return linear


def cpu_baseline_layer(case, act_bits=8, rot=0, asym=False, target_seconds=12.0, layer=0):
    """The oracle on a bounded sample of token rows (all N, all K) of one layer."""
    import oracle
    linear = _oracle_linear(case, layer, act_bits, rot, asym)
    threads = oracle.num_threads()
    probe_rows = 64
    x = case.x_rows(0, probe_rows)
    t0 = time.perf_counter()
    linear(x)
    per_row = (time.perf_counter() - t0) / probe_rows
    rows = int(min(case.M, max(probe_rows, target_seconds / per_row)))
    rows -= rows % 64
    x = case.x_rows(0, rows)
    reps, dt = 0, 0.0
    while reps == 0 or (dt < 0.8 * target_seconds and reps < 50):
        t0 = time.perf_counter()
        linear(x)
        dt += time.perf_counter() - t0
        reps += 1
    tops = 2.0 * reps * rows * case.N * case.K / dt / 1e12
    # the same oracle on one thread, on a sixteenth of the sample
    one_rows = max(64, rows // 16 - (rows // 16) % 64)
    x1 = case.x_rows(0, one_rows)
    oracle.set_num_threads(1)
    t0 = time.perf_counter()
    linear(x1)
    dt1 = time.perf_counter() - t0
    oracle.set_num_threads(threads)
    one_thread = 2.0 * one_rows * case.N * case.K / dt1 / 1e12
    return {"value": tops, "unit": "TOPS", "cores": threads, "kind": "oracle",
            "one_thread": {"value": one_thread, "rows": one_rows, "seconds": dt1},
            "sample": f"first {rows} of {case.M} token rows x all N={case.N} x K={case.K} of "
                      f"layer {case.name} (quantize + int32 GEMM + epilogue), {reps} passes in "
                      f"{dt:.2f} s, OpenMP over rows",
            "seconds": dt}


def cpu_baseline_sweep(cases, act_bits, rot, asym, target_seconds=20.0):
    """The oracle on a row sample of one layer of each distinct (shape, weight bits) class of
    the sweep; the classes' rates are combined with the number of layers of each class."""
    import oracle
    classes = {}
    for i, c in enumerate(cases):
        classes.setdefault((c.K, c.N, c.bits, c.epi), []).append(i)
    threads = oracle.num_threads()
    t_start = time.perf_counter()
    per_class, total_ops, total_seconds, parts = [], 0.0, 0.0, []
    budget = target_seconds / len(classes)
    for (K, N, bits, epi), idx in classes.items():
        case, layer = cases[idx[0]], idx[0]
        linear = _oracle_linear(case, layer, act_bits, rot, asym)
        x = case.x_rows(0, 64)
        t0 = time.perf_counter()
        linear(x)
        per_row = (time.perf_counter() - t0) / 64
        rows = int(min(case.M, max(64, 0.7 * budget / per_row)))
        rows -= rows % 64
        x = case.x_rows(0, rows)
        t0 = time.perf_counter()
        linear(x)
        dt = time.perf_counter() - t0
        sec_per_layer = dt / rows * case.M           # extrapolated to all M rows
        total_seconds += sec_per_layer * len(idx)
        total_ops += 2.0 * case.M * N * K * len(idx)
        per_class.append({"K": K, "N": N, "weight_bits": bits, "epilogue": epi, "layers": len(idx),
                          "rows": rows, "seconds": round(dt, 3),
                          "tops": round(2.0 * rows * N * K / dt / 1e12, 5)})
        parts.append(f"{rows} rows of {case.name}")
    return {"value": total_ops / total_seconds / 1e12, "unit": "TOPS", "cores": threads,
            "kind": "oracle",
            "sample": "one layer of each of the sweep's " + str(len(classes)) + " (shape, weight bits) "
                      "classes on its first rows (all N, all K; quantize + int32 GEMM + epilogue; "
                      "OpenMP over rows): " + ", ".join(parts) + "; rows are independent, so each "
                      "class's time is scaled to M = " + str(cases[0].M) + " rows and weighted by its "
                      "number of layers (extrapolated)",
            "extrapolated_seconds_per_step": round(total_seconds, 1),
            "classes": per_class, "seconds": round(time.perf_counter() - t_start, 2)}


# ---- the workloads ---------------------------------------------------------------------------------

class Layer:
    """Device buffers of one quantized linear."""

    def __init__(self, case, x, ws, Y, layer_index=0, rot=0, asym=False):
        import torch
        from paper_2503_06545_amd import binding as qc
        self.case, self.x, self.ws, self.Y = case, x, ws, Y
        self.W = torch.from_numpy(case.weight(layer_index)).cuda()
        self.bias = torch.from_numpy(case.bias(layer_index)).cuda()
        self.pw = qc.pack_weight_t(self.W, case.bits, rot)
        self.row_sums = qc.weight_row_sums_t(self.pw) if asym else None
        self.epi = qc.EPI[case.epi]
        self.ops = 2.0 * case.M * case.N * case.K


class Bench:
    """Everything that is shared between the workloads of one run."""

    def __init__(self, variant, roofs, graph=False):
        self.graph = graph
        import torch
        from paper_2503_06545_amd import binding as qc
        from paper_2503_06545_amd import synth
        self.torch, self.qc, self.synth = torch, qc, synth
        var = VARIANTS[variant]
        self.variant = variant
        self.act_bits, self.rot, self.asym = var["act_bits"], var.get("rot", 0), var.get("asym", False)
        self.roofs = roofs
        self.traffic, self.traffic_commit = traffic_table()
        self.stream = torch.cuda.current_stream().cuda_stream
        # The latent change does not depend on the linear: a step issues it on a second stream
        # (default priority) so that this HBM-bound reduction runs beside the GEMM.
        self.side = torch.cuda.Stream()
        self.x_dev = {}       # (K, post_gelu) -> device activations, the longest M asked for
        cur_h, prev_h = synth.latent_pair(seed=0)
        self.cur, self.prev = torch.from_numpy(cur_h).cuda(), torch.from_numpy(prev_h).cuda()
        self.n_lat = self.cur.numel()
        self.dws = qc.latent_delta_workspace_t(self.n_lat)
        self.out3 = torch.empty(3, dtype=torch.float32, device="cuda")

    # -- inputs: the single-layer configurations are row prefixes of the sweep's tensors (the
    #    generator is keyed by row block), so one tensor per (K, distribution) serves them all
    def activations(self, case):
        import dataclasses
        import numpy as np
        key = (case.K, case.post_gelu, case.outliers, case.seed)
        if key not in self.x_dev or self.x_dev[key].shape[0] < case.M:
            bits = dataclasses.replace(case, x_dtype="bf16").x()
            self.x_dev[key] = self.torch.from_numpy(bits.view(np.int16)).cuda().view(self.torch.bfloat16)
        return self.x_dev[key][:case.M]

    def gemm_kernel_name(self, case):
        """Which of the GEMM's two kernels the library takes for this layer."""
        which = self.qc.qc_debug_gemm_kernel(case.M, case.K, case.N, case.bits)
        return "gemm_resident_kernel" if which == 2 else "gemm_kernel"

    def check(self, st):
        if st != self.qc.QC_OK:
            raise self.qc.QcError(st, "bench step")

    # -- the calls
    def qlinear(self, L):
        qc, c = self.qc, L.case
        tail = (c.bits, c.N, L.bias.data_ptr(), L.epi, L.Y.data_ptr(), qc.QC_OUT_BF16,
                L.ws.data_ptr(), L.ws.numel(), self.stream)
        head = (L.x.data_ptr(), qc.QC_BF16, c.M, c.K)
        if self.asym:
            self.check(qc.qc_qlinear_asym(*head, self.act_bits, L.pw.blob.data_ptr(), L.pw.scale.data_ptr(),
                                          L.row_sums.data_ptr(), *tail))
        elif self.rot:
            self.check(qc.qc_qlinear_rot(*head, self.act_bits, self.rot, L.pw.blob.data_ptr(),
                                         L.pw.scale.data_ptr(), *tail))
        elif self.act_bits != 8:
            self.check(qc.qc_qlinear_act_bits(*head, self.act_bits, L.pw.blob.data_ptr(),
                                              L.pw.scale.data_ptr(), *tail))
        else:
            self.check(qc.qc_qlinear(*head, L.pw.blob.data_ptr(), L.pw.scale.data_ptr(), *tail))

    def quant_stage(self, L, x=None):
        qc, c = self.qc, L.case
        head = ((L.x if x is None else x).data_ptr(), qc.QC_BF16, c.M, c.K)
        tail = (L.ws.data_ptr(), L.ws.numel(), self.stream)
        if self.asym:
            self.check(qc.qc_qlinear_asym_quant(*head, self.act_bits, *tail))
        elif self.rot:
            self.check(qc.qc_qlinear_quant_rot(*head, self.act_bits, self.rot, *tail))
        else:
            self.check(qc.qc_qlinear_quant_bits(*head, self.act_bits, *tail))

    def gemm_stage(self, L):
        qc, c = self.qc, L.case
        tail = (c.bits, c.N, L.bias.data_ptr(), L.epi, L.Y.data_ptr(), qc.QC_OUT_BF16, self.stream)
        if self.asym:
            self.check(qc.qc_qlinear_asym_gemm(L.ws.data_ptr(), L.ws.numel(), c.M, c.K,
                                               L.pw.blob.data_ptr(), L.pw.scale.data_ptr(),
                                               L.row_sums.data_ptr(), *tail))
        else:
            self.check(qc.qc_qlinear_gemm(L.ws.data_ptr(), L.ws.numel(), c.M, c.K,
                                          L.pw.blob.data_ptr(), L.pw.scale.data_ptr(), *tail))

    def delta_stage(self, on=None, pair=None):
        a, b = pair if pair is not None else (self.cur, self.prev)
        self.check(self.qc.qc_latent_delta(a.data_ptr(), b.data_ptr(), self.n_lat, self.out3.data_ptr(),
                                           self.dws.data_ptr(), self.dws.numel(),
                                           self.stream if on is None else on))

    def pack_stage(self, L):
        qc, c = self.qc, L.case
        if self.rot:
            self.check(qc.qc_pack_weight_rot(L.W.data_ptr(), c.N, c.K, c.bits, self.rot,
                                             L.pw.blob.data_ptr(), L.pw.scale.data_ptr(), self.stream))
        else:
            self.check(qc.qc_pack_weight(L.W.data_ptr(), c.N, c.K, c.bits, L.pw.blob.data_ptr(),
                                         L.pw.scale.data_ptr(), self.stream))

    # -- rooflines
    def mfma_roofline(self, name, kernel_name, ops, gemm_us, launches):
        tops = ops / (gemm_us * 1e-6) / 1e12
        r = {"bound": "mfma", "kernel": kernel_name, "achieved": round(tops, 1),
             "peak": PEAK_INT8_TOPS, "unit": "TOP/s", "frac": round(tops / PEAK_INT8_TOPS, 4),
             "traffic": self.traffic.get(name, {}).get("gemm") if self.variant == "a8" else None,
             "traffic_source": ("profiles/hbm_traffic_per_launch.txt: rocprofv3 --pmc FETCH_SIZE / "
                                "WRITE_SIZE passes of this script at commit " + str(self.traffic_commit) +
                                ", not a measurement of this run"),
             "ops_per_launch": ops / launches, "launches_per_step": launches,
             "avg_launch_us": round(gemm_us / launches, 2)}
        rand, fed = self.roofs.get("mfma_16x16x64_random_tops"), self.roofs.get("mfma_16x16x64_gemm_traffic_tops")
        r["achievable"] = {
            "mfma_registers_only_random_operands": rand,
            "mfma_with_the_gemms_operand_traffic": fed,
            "note": "measured in this run by bench/qc_roofs: the v_mfma_i32_16x16x64_i8 loop on random "
                    "int8 operands held in registers, and the same loop fed 0.5 LDS fragment reads "
                    "and 384 B from L2 per 32 K multiply-adds (the GEMM's proportions; a yardstick, "
                    "not a bound)"}
        r["frac_of_achievable"] = round(tops / rand, 4) if rand else None
        r["frac_of_traffic_yardstick"] = round(tops / fed, 4) if fed else None
        return r

    def hbm_entry(self, bytes_per_launch, us, roof_key="hbm_read2_write1_gbs", traffic=None):
        gbs = bytes_per_launch / (us * 1e-6) / 1e9
        roof = self.roofs.get(roof_key)
        return {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(gbs / PEAK_HBM_GBS, 4), "bytes_per_launch": bytes_per_launch,
                "avg_launch_us": round(us, 2), "traffic": traffic,
                "achievable": roof, "achievable_is": roof_key + " of bench/qc_roofs, this run",
                "frac_of_achievable": round(gbs / roof, 4) if roof else None}

    # -- one single-layer configuration: qc_qlinear + qc_latent_delta on a second stream
    def run_single(self, name, steps, warmup, with_cold=True):
        torch, qc, synth = self.torch, self.qc, self.synth
        case = {"qkv256": synth.QKV_256, "fc1_512": synth.FC1_512, "fc2_512_w8": synth.FC2_512_W8,
                "fc2_512_w4": synth.FC2_512_W4}[name]
        x = self.activations(case)
        ws = (qc.qlinear_asym_workspace_t if self.asym else qc.qlinear_workspace_t)(case.M, case.K, case.N)
        Y = torch.empty(case.M * case.N, dtype=torch.bfloat16, device="cuda")
        L = Layer(case, x, ws, Y, 0, self.rot, self.asym)

        def step():
            self.qlinear(L)
            self.delta_stage(self.side.cuda_stream)

        preload(step)
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        with PowerSampler() as sampler:
            t0 = time.perf_counter()
            for _ in range(steps):
                step()
            torch.cuda.synchronize()
            ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
        device = sampler.summary()
        value = L.ops / (ms_per_step * 1e-3) / 1e12

        batch = 20
        rounds = max(3, min(steps, 400) // batch)
        preload(step, 0.1)
        quant = batch_times_us(lambda: self.quant_stage(L), batch, rounds)
        gemm = batch_times_us(lambda: self.gemm_stage(L), batch, rounds)
        delta = batch_times_us(self.delta_stage, batch, rounds)
        pack = batch_times_us(lambda: self.pack_stage(L), 1, 5)
        tr = self.traffic.get(name, {}) if self.variant == "a8" else {}
        quant_bytes = case.M * case.K * 3 + 4 * case.M
        delta_bytes = 2 * self.n_lat * 4 + 12
        whole_us = quant["avg_us"] + gemm["avg_us"]
        res = {
            "workload": DESCRIBE[name], "M": case.M, "K": case.K, "N": case.N,
            "weight_bits": case.bits, "epilogue": case.epi,
            "steps": steps, "warmup": warmup, "preload_s": PRELOAD_SECONDS,
            "ms_per_step": round(ms_per_step, 5), "value": round(value, 2), "unit": "TOPS",
            "frac_of_peak": round(value / PEAK_INT8_TOPS, 4),
            "device": device,
            "roofline": self.mfma_roofline(name, f"{self.gemm_kernel_name(case)}<{case.bits}, bf16, {case.epi}>", L.ops,
                                           gemm["avg_us"], 1),
            "kernels": {
                "quant_act": self.hbm_entry(quant_bytes, quant["avg_us"], traffic=tr.get("quant")),
                "latent_delta": dict(self.hbm_entry(delta_bytes, delta["avg_us"], "hbm_read_gbs",
                                                    traffic=tr.get("delta")),
                                     note="two launches per call; the same 33.5 MB pair on every call (it "
                                          "fits the 256 MB Infinity Cache, but the kernel's non-temporal "
                                          "loads do not leave it there)"),
                "pack_weight_offline": {"avg_launch_us": round(pack["avg_us"], 2)},
                # quantization + GEMM + epilogue of the layer, without the latent delta
                "qlinear_whole_call": {
                    "achieved": round(L.ops / (whole_us * 1e-6) / 1e12, 1), "peak": PEAK_INT8_TOPS,
                    "unit": "TOP/s", "frac": round(L.ops / (whole_us * 1e-6) / 1e12 / PEAK_INT8_TOPS, 4),
                    "avg_us": round(whole_us, 2)},
            },
        }
        if with_cold:
            # The same two kernels on inputs that are cold in the L2s and the 256 MB Infinity
            # Cache: each launch takes the next of enough distinct copies of its input to exceed
            # 320 MB (a layer whose activations are larger than that is cold anyway).
            turn = [0]
            copies = max(2, -(-(320 << 20) // (x.numel() * 2)))
            xs = [x] + [x.clone() for _ in range(copies - 1)]

            def quant_cold():
                self.quant_stage(L, xs[turn[0] % copies])
                turn[0] += 1
            qcold = batch_times_us(quant_cold, copies, max(3, 60 // copies))
            del xs
            pairs = -(-(320 << 20) // (2 * self.n_lat * 4))
            lat = [(self.cur, self.prev)] + [(self.cur.clone(), self.prev.clone()) for _ in range(pairs - 1)]

            def delta_cold():
                self.delta_stage(pair=lat[turn[0] % pairs])
                turn[0] += 1
            dcold = batch_times_us(delta_cold, pairs, 8)
            del lat
            res["kernels"]["quant_act"]["cold"] = dict(
                self.hbm_entry(quant_bytes, qcold["avg_us"]),
                note="each launch reads the next of enough distinct input copies to exceed 320 MB")
            cold_roof_us = self.roofs.get("read_32mib_cold_us")
            res["kernels"]["latent_delta"]["cold"] = dict(
                self.hbm_entry(delta_bytes, dcold["avg_us"], "hbm_read_gbs"),
                read_only_kernel_same_bytes_us=cold_roof_us,
                frac_of_read_only_kernel=round(cold_roof_us / dcold["avg_us"], 4) if cold_roof_us else None,
                note="each call takes the next of enough distinct latent pairs to exceed 320 MB; "
                     "read_only_kernel_same_bytes_us is bench/qc_roofs' single launch that only reads "
                     "two cold 16 MiB buffers, timed the same way (launch boundary included)")
        del L, Y, ws
        torch.cuda.empty_cache()
        return res, case

    # -- the 28-block sweep
    def run_sweep(self, steps, warmup):
        torch, qc, synth = self.torch, self.qc, self.synth
        cases = synth.stdit_block_layers()
        M = cases[0].M
        maxK, maxN = max(c.K for c in cases), max(c.N for c in cases)
        ws = (qc.qlinear_asym_workspace_t if self.asym else qc.qlinear_workspace_t)(M, maxK, maxN)
        Y = torch.empty(M * maxN, dtype=torch.bfloat16, device="cuda")
        layers = [Layer(c, self.activations(c), ws, Y, i, self.rot, self.asym) for i, c in enumerate(cases)]

        def step():
            for L in layers:
                self.qlinear(L)

        eager_step = step
        if self.graph:
            # The 224 launches of a step recorded once into a HIP graph (no entry point
            # allocates, clears or needs a set-up call, so the calls can be captured as they
            # are) and replayed: the step then costs one submission instead of 224.
            torch.cuda.synchronize()
            g, cap = torch.cuda.CUDAGraph(), torch.cuda.Stream()
            main_stream, self.stream = self.stream, cap.cuda_stream   # the calls go to the capturing stream
            with torch.cuda.graph(g, stream=cap):
                eager_step()
            self.stream = main_stream
            step = g.replay
        preload(step)
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        with PowerSampler() as sampler:
            t0 = time.perf_counter()
            for _ in range(steps):
                step()
            torch.cuda.synchronize()
            ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
        device = sampler.summary()
        ops = sum(L.ops for L in layers)
        value = ops / (ms_per_step * 1e-3) / 1e12

        rounds = 3
        quant = batch_times_us(lambda: [self.quant_stage(L) for L in layers], 1, rounds)
        gemm = batch_times_us(lambda: [self.gemm_stage(L) for L in layers], 1, rounds)
        pack = batch_times_us(lambda: [self.pack_stage(L) for L in layers], 1, 2)
        # the GEMM by class of layer (shape, weight bits): all layers of a class, back to back
        by_class = {}
        for L in layers:
            by_class.setdefault((L.case.name.split("_")[1], L.case.bits), []).append(L)
        classes = []
        for (kind, bits), ls in by_class.items():
            t = batch_times_us(lambda: [self.gemm_stage(L) for L in ls], 1, 3)
            q = batch_times_us(lambda: [self.quant_stage(L) for L in ls], 1, 2)
            c = ls[0].case
            tops = sum(L.ops for L in ls) / (t["avg_us"] * 1e-6) / 1e12
            qbytes = (c.M * c.K * 3 + 4 * c.M)
            classes.append({"layer": kind, "K": c.K, "N": c.N, "weight_bits": bits, "layers": len(ls),
                            "gemm_kernel": self.gemm_kernel_name(c),
                            "gemm_avg_launch_us": round(t["avg_us"] / len(ls), 1),
                            "gemm_tops": round(tops, 1), "gemm_frac": round(tops / PEAK_INT8_TOPS, 4),
                            "quant_avg_launch_us": round(q["avg_us"] / len(ls), 1),
                            "quant_gbs": round(qbytes / (q["avg_us"] / len(ls) * 1e-6) / 1e9, 1)})
        n = len(layers)
        quant_bytes = sum(c.M * c.K * 3 + 4 * c.M for c in cases)
        whole_us = quant["avg_us"] + gemm["avg_us"]
        tr = self.traffic.get("sweep28", {}) if self.variant == "a8" else {}
        res = {
            "workload": DESCRIBE["sweep28"], "M": M, "layers": n,
            "w4_layers": sum(c.bits == 4 for c in cases),
            "steps": steps, "warmup": warmup, "preload_s": PRELOAD_SECONDS,
            "ms_per_step": round(ms_per_step, 4), "value": round(value, 2), "unit": "TOPS",
            "frac_of_peak": round(value / PEAK_INT8_TOPS, 4), "device": device,
            "roofline": self.mfma_roofline("sweep28", "gemm_resident_kernel | gemm_kernel<8|4, bf16, none|gelu_tanh> (112 launches)",
                                           ops, gemm["avg_us"], n),
            "kernels": {
                "quant_act": self.hbm_entry(quant_bytes / n, quant["avg_us"] / n, traffic=tr.get("quant")),
                "pack_weight_offline": {"avg_launch_us": round(pack["avg_us"] / n, 2)},
                "qlinear_whole_call": {
                    "achieved": round(ops / (whole_us * 1e-6) / 1e12, 1), "peak": PEAK_INT8_TOPS,
                    "unit": "TOP/s", "frac": round(ops / (whole_us * 1e-6) / 1e12 / PEAK_INT8_TOPS, 4),
                    "avg_us": round(whole_us / n, 2)},
                "gemm_by_layer_class": classes,
            },
        }
        del layers, Y, ws
        torch.cuda.empty_cache()
        return res, cases


def library_int8_gemm(bench, cases):
    """The vendor library's int8 GEMM (torch._int_mm: int8 x int8 -> int32, nothing fused) on the
    distinct (M, K, N) of the workload, fed with the very codes this library's quantizers produce
    for the workload's activations and weights (operand values decide how much power an MFMA
    draws), after the same 0.3 s of load; and on one large square, with such codes and with
    uniform random bytes.  Only a yardstick: it shows what rate the library's own kernels hold on
    this chip under its power cap; its output is 4 bytes per element where the path's epilogue
    writes 2."""
    import torch
    qc = bench.qc

    def timed(a, b):
        M, K = a.shape
        N = b.shape[1]
        try:
            torch._int_mm(a, b)
        except RuntimeError as e:
            return {"error": str(e)[:120]}
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < PRELOAD_SECONDS:
            torch._int_mm(a, b)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        iters = 30
        e0.record()
        for _ in range(iters):
            torch._int_mm(a, b)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / iters
        tops = 2.0 * M * N * K / (us * 1e-6) / 1e12
        return {"avg_us": round(us, 1), "tops": round(tops, 1), "frac": round(tops / PEAK_INT8_TOPS, 4)}

    def codes(x_bf16, w_f32, bits):
        a = qc.quant_act_t(x_bf16, 8)[0]
        b = qc.unpack_weight_codes_t(qc.pack_weight_t(w_f32, bits))
        return a, b.t()

    out = {"what": "torch._int_mm, int32 out; operands: the codes of the workload's own activations "
                   "and weights", "shapes": {}}
    seen = set()
    for layer, c in enumerate(cases):
        if (c.M, c.K, c.N) in seen:
            continue
        seen.add((c.M, c.K, c.N))
        a, b = codes(bench.activations(c), torch.from_numpy(c.weight(layer)).cuda(), c.bits)
        out["shapes"][f"{c.M}x{c.K}x{c.N}"] = dict(timed(a, b), weight_bits=c.bits)
        del a, b
    n = 8192
    gen = torch.Generator(device="cuda").manual_seed(0)
    x = torch.randn((n, n), device="cuda", generator=gen).to(torch.bfloat16)
    w = torch.randn((n, n), device="cuda", generator=gen) * 0.02
    a, b = codes(x, w, 8)
    out["square_8192"] = {"codes_of_normal_data": timed(a, b)}
    a = torch.randint(-127, 128, (n, n), dtype=torch.int8, device="cuda", generator=gen)
    b = torch.randint(-127, 128, (n, n), dtype=torch.int8, device="cuda", generator=gen).t()
    out["square_8192"]["uniform_random_bytes"] = timed(a, b)
    # the same square through this library's GEMM stage (bf16 out, no activation)
    pw = qc.pack_weight_t(w, 8)
    ws = qc.qlinear_workspace_t(n, n, n)
    bias = torch.zeros(n, device="cuda")
    y = qc.qlinear_t(x, pw, bias, "none", "bf16", workspace=ws)
    args = (ws.data_ptr(), ws.numel(), n, n, pw.blob.data_ptr(), pw.scale.data_ptr(), 8, n,
            bias.data_ptr(), qc.QC_EPI_NONE, y.data_ptr(), qc.QC_OUT_BF16, bench.stream)
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < PRELOAD_SECONDS:
        bench.check(qc.qc_qlinear_gemm(*args))
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(30):
        bench.check(qc.qc_qlinear_gemm(*args))
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / 30
    tops = 2.0 * n ** 3 / (us * 1e-6) / 1e12
    out["square_8192"]["qc_qlinear_gemm"] = {"avg_us": round(us, 1), "tops": round(tops, 1),
                                             "frac": round(tops / PEAK_INT8_TOPS, 4)}
    del a, b, x, w, y, ws
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", choices=WORKLOADS, default="sweep28",
                    help="the headline; the default sweep also reports the single-layer "
                         "configurations under `configs`")
    ap.add_argument("--variant", choices=tuple(VARIANTS), default="a8",
                    help="activation quantizer: a8 (default), a6 / a4 (lower bit-widths), rot128 "
                         "(Walsh-Hadamard rotation of 128-column blocks fused in), asym (zero "
                         "point per token)")
    ap.add_argument("--graph", action="store_true",
                    help="sweep28: record the step's launches once into a HIP graph and time replays")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true",
                    help="sweep28 only: skip the single-layer configurations")
    ap.add_argument("--no-roofs", action="store_true", help="do not run bench/qc_roofs first")
    ap.add_argument("--library-gemm", action="store_true",
                    help="also time the int8 GEMM of the library that ships with ROCm (through "
                         "torch._int_mm, int32 output, no scales / bias / GELU) on the workload's "
                         "shapes: a yardstick for the power-limited MFMA rate, not a part of the path")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a few plain 256 MiB device copies, as the reference kernel "
                         "for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); the path shards by token "
              "rows without any exchange between GPUs", file=sys.stderr)
        return 2

    # the roofs first: the child process has the GPU to itself and is gone before torch starts
    roofs = {} if args.no_roofs else measured_roofs()

    import torch
    from paper_2503_06545_amd import binding as qc

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    qc.lib()  # fail loudly if libqc.so is missing

    sweep = args.workload == "sweep28"
    steps = args.steps if args.steps is not None else (20 if sweep else 300)
    warmup = args.warmup if args.warmup is not None else (5 if sweep else 100)
    bench = Bench(args.variant, roofs, args.graph)

    configs = {}
    if sweep:
        head, cases = bench.run_sweep(steps, warmup)
        if not args.no_configs:
            for name in SINGLE:
                # about a quarter of a second of timed steps each, whatever --steps says
                per_step_ms = {"qkv256": 0.075, "fc1_512": 0.37, "fc2_512_w8": 0.45, "fc2_512_w4": 0.42}[name]
                sub_steps = max(50, int(250 / per_step_ms))
                configs[name], _ = bench.run_single(name, sub_steps, sub_steps // 4,
                                                    with_cold=name in ("qkv256", "fc1_512"))
    else:
        head, case = bench.run_single(args.workload, steps, warmup)
        cases = [case]

    library = library_int8_gemm(bench, cases) if args.library_gemm else None

    if args.calibration_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()

    result = {
        "metric": "quantized-linear int8 TOPS, whole qc_qlinear" +
                  ("" if sweep else " + qc_latent_delta") + " step, 1 MI355X",
        "value": head["value"],
        "unit": "TOPS",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8 (int32 accumulate; bf16 in/out, fp32 scales)",
        "data": "synthetic",
        "config": {"workload": head["workload"], "name": args.workload, "variant": args.variant,
                   "activation_quantizer": VARIANT_TEXT[args.variant],
                   "layers": len(cases), "w4_layers": sum(c.bits == 4 for c in cases),
                   "M": cases[0].M, "seed": cases[0].seed,
                   "preload_s": PRELOAD_SECONDS,
                   "offline_not_in_step": "qc_pack_weight",
                   "streams": "qc_qlinear on the current stream" +
                              ("" if sweep else ", qc_latent_delta on a second one")},
        "device": dict(name=torch.cuda.get_device_name(0), **head["device"]),
        "roofline": head["roofline"],
        "kernels": head["kernels"],
        "achievable_roofs": roofs,
        "provenance": provenance(),
    }
    if not sweep:
        c = cases[0]
        result["config"].update({"K": c.K, "N": c.N, "weight_bits": c.bits, "epilogue": c.epi})
    if configs:
        result["configs"] = configs
    if library is not None:
        result["library_int8_gemm"] = library
    if not args.no_cpu_baseline:
        if sweep:
            result["cpu_baseline"] = cpu_baseline_sweep(cases, bench.act_bits, bench.rot, bench.asym)
        else:
            result["cpu_baseline"] = cpu_baseline_layer(cases[0], bench.act_bits, bench.rot, bench.asym)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
