#!/usr/bin/env python3
"""Benchmark of the quantized-linear hot path on one MI355X.

A step is one pass of the per-step hot path over one batch of seeded synthetic input.  The
default workload is the STDiT QKV projection of a 256x256 video (X bf16 [16384, 1152],
W int8 [3456, 1152], bf16 out): qc_qlinear (per-token activation quantization + int8 MFMA
GEMM + dequant/bias epilogue) followed by qc_latent_delta on two [16, 4, 16, 64, 64] float
latents.  `--workload` selects the other STDiT layers (fc1+GELU, fc2 with int8 or int4
weights) or the 28-block sweep (112 qc_qlinear calls, per-layer bit-width from the seeded
importance mask); `--variant` selects how the activations are quantized (lower bit-widths,
rotation fused in, or the asymmetric form), the GEMM kernel being the same.  Weights are packed once before the timed region (an offline step of the
method); the packing time is reported beside the result.  Inputs are resident in HBM when
timing starts.

Prints ONE JSON line.  `value` = integer ops (2*M*N*K per layer) of the step divided by the
step time.  `roofline` describes the dominant kernel (the GEMM), timed with HIP events around
batches of its launches; `kernels` adds the HBM-bound kernels; `cpu_baseline` is the CPU
oracle timed on this host's cores on a bounded row sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0   # MI355X dense int8 MFMA, 5.0 POP/s
PEAK_HBM_GBS = 8000.0     # MI355X HBM3E, 8 TB/s

# Bytes per launch between L2 and the fabric (Infinity Cache / HBM) from `rocprofv3 --pmc
# FETCH_SIZE` / `--pmc WRITE_SIZE` runs of this script, scaled by the same counters on a plain
# 256 MiB copy (profiles/bench_<workload>_rocprofv3.txt).
MEASURED_TRAFFIC_BYTES = {
    "qkv256": {"gemm": 165.5e6, "quant": 56.9e6, "delta": 33.6e6},
    "fc1_512": {"gemm": 852.5e6, "quant": 226.9e6, "delta": 33.6e6},
    "fc2_512_w8": {"gemm": 1304.7e6, "quant": 906.3e6, "delta": 33.6e6},
    "fc2_512_w4": {"gemm": 814.8e6, "quant": 906.3e6, "delta": 33.6e6},
}

WORKLOADS = ("qkv256", "fc1_512", "fc2_512_w8", "fc2_512_w4", "sweep28")
# How the activations are quantized: the spec form (symmetric int8 per token), the lower
# activation bit-widths of Eq. (8), the rotation fused into the quantization, or the printed
# asymmetric form of Eq. (3)-(4).  The GEMM is the same kernel in all of them.
VARIANTS = {"a8": dict(act_bits=8), "a6": dict(act_bits=6), "a4": dict(act_bits=4),
            "rot128": dict(act_bits=8, rot=128), "asym": dict(act_bits=8, asym=True)}


def batch_times_us(fn, batch, rounds):
    """Average duration of one fn() from HIP events around batches of back-to-back calls
    (a batch keeps the GPU loaded and amortises the dispatch gap that an event pair around a
    single launch would include)."""
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


def cpu_baseline(case, act_bits=8, rot=0, asym=False, target_seconds=15.0):
    """The oracle as it stands on a bounded sample of token rows (all N, all K)."""
    import oracle
    W, b = case.weight(), case.bias()
    qw, sw = oracle.quant_weight_rot(W, case.bits, rot) if rot else oracle.quant_weight(W, case.bits)
    epi = {"none": oracle.EPI_NONE, "gelu_tanh": oracle.EPI_GELU_TANH,
           "gelu_erf": oracle.EPI_GELU_ERF}[case.epi]

    def linear(x):
        if asym:
            return oracle.qlinear_asym(x, qw, sw, b, epi, act_bits)
        if rot:
            return oracle.qlinear_rot(x, qw, sw, rot, b, epi, act_bits)
        return oracle.qlinear(x, qw, sw, b, epi, act_bits)

    threads = oracle.num_threads()
    probe_rows = 64
    x = case.x_rows(0, probe_rows)
    t0 = time.perf_counter()
    linear(x)
    per_row = (time.perf_counter() - t0) / probe_rows
    rows = int(min(case.M, max(probe_rows, target_seconds / per_row)))
    rows -= rows % 64
    x = case.x_rows(0, rows)
    # about 10 s of wall time on all host cores: the sample is repeated if one pass is shorter
    reps, dt = 0, 0.0
    while reps == 0 or (dt < 10.0 and reps < 50):
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    # the GPU needs some tens of milliseconds of load before its clocks have ramped up; the
    # default warm-up is ~0.1 s of steps
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", choices=WORKLOADS, default="qkv256")
    ap.add_argument("--variant", choices=tuple(VARIANTS), default="a8",
                    help="activation quantizer: a8 (default), a6 / a4 (lower bit-widths), rot128 "
                         "(Walsh-Hadamard rotation of 128-column blocks fused in), asym (zero "
                         "point per token)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a few plain 256 MiB device copies, as the reference kernel "
                         "for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); the path shards by token "
              "rows without any exchange between GPUs", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2503_06545_amd import binding as qc
    from paper_2503_06545_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    qc.lib()  # fail loudly if libqc.so is missing

    def to_dev_bf16(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)

    # ---- workload ------------------------------------------------------------------------
    sweep = args.workload == "sweep28"
    if sweep:
        cases = synth.stdit_block_layers()
        describe = ("28 STDiT blocks x (QKV 1152->3456, out 1152->1152, fc1 1152->4608 + GELU, "
                    "fc2 4608->1152), M = 131072 tokens (CFG batch 2 at 512x512), bf16 in/out, "
                    "per-layer weight bit-width from the seeded mask")
        default_steps, default_warmup = 20, 4
    else:
        case0 = {"qkv256": synth.QKV_256, "fc1_512": synth.FC1_512, "fc2_512_w8": synth.FC2_512_W8,
                 "fc2_512_w4": synth.FC2_512_W4}[args.workload]
        cases = [case0]
        describe = {
            "qkv256": "STDiT QKV projection 256x256, the headline configuration: X bf16 [16384,1152] "
                      "N(0,1) with 12 outlier columns x20, W8A8 [3456,1152], bias, bf16 out",
            "fc1_512": "STDiT MLP fc1 + GELU(tanh) 512x512: X bf16 "
                       "[65536,1152], W8A8 [4608,1152], bf16 out",
            "fc2_512_w8": "STDiT MLP fc2 512x512: X bf16 [65536,4608] "
                          "post-GELU, W8A8 [1152,4608], bf16 out",
            "fc2_512_w4": "STDiT MLP fc2 512x512: X bf16 [65536,4608] "
                          "post-GELU, W4A8 [1152,4608] int4 weights, bf16 out",
        }[args.workload] + "; + latent delta on 2 x [16,4,16,64,64] fp32"
        scale = max(1, (case0.M * case0.N * case0.K) // (16384 * 3456 * 1152))
        default_steps, default_warmup = max(200, 3000 // scale), max(100, 1000 // scale)
    steps = args.steps if args.steps is not None else default_steps
    warmup = args.warmup if args.warmup is not None else default_warmup

    # one activation tensor per distinct (K, distribution), shared by the layers that use it
    x_cache, layers = {}, []
    M = cases[0].M
    maxK = max(c.K for c in cases)
    maxN = max(c.N for c in cases)
    var = VARIANTS[args.variant]
    act_bits, rot, asym = var["act_bits"], var.get("rot", 0), var.get("asym", False)
    ws = (qc.qlinear_asym_workspace_t if asym else qc.qlinear_workspace_t)(M, maxK, maxN)
    Y = torch.empty(M * maxN, dtype=torch.bfloat16, device="cuda")
    for i, c in enumerate(cases):
        key = (c.K, c.post_gelu, c.outliers)
        if key not in x_cache:
            x_cache[key] = to_dev_bf16(c.x())
        layers.append(Layer(c, x_cache[key], ws, Y, layer_index=i, rot=rot, asym=asym))
    w4_layers = sum(c.bits == 4 for c in cases)

    cur_h, prev_h = synth.latent_pair(seed=0)
    cur, prev = torch.from_numpy(cur_h).cuda(), torch.from_numpy(prev_h).cuda()
    n_lat = cur.numel()
    dws = qc.latent_delta_workspace_t(n_lat)
    out3 = torch.empty(3, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    # The latent change does not depend on the linear: the step issues it on a second stream
    # (default priority) so that this HBM-bound reduction runs beside the GEMM.  Successive
    # calls on that stream share one workspace and are ordered by the stream itself.
    side = torch.cuda.Stream()
    side_stream = side.cuda_stream

    def check(st):
        if st != qc.QC_OK:
            raise qc.QcError(st, "bench step")

    def qlinear(L):
        c = L.case
        tail = (c.bits, c.N, L.bias.data_ptr(), L.epi, L.Y.data_ptr(), qc.QC_OUT_BF16,
                L.ws.data_ptr(), L.ws.numel(), stream)
        head = (L.x.data_ptr(), qc.QC_BF16, c.M, c.K)
        if asym:
            check(qc.qc_qlinear_asym(*head, act_bits, L.pw.blob.data_ptr(), L.pw.scale.data_ptr(),
                                     L.row_sums.data_ptr(), *tail))
        elif rot:
            check(qc.qc_qlinear_rot(*head, act_bits, rot, L.pw.blob.data_ptr(),
                                    L.pw.scale.data_ptr(), *tail))
        elif act_bits != 8:
            check(qc.qc_qlinear_act_bits(*head, act_bits, L.pw.blob.data_ptr(),
                                         L.pw.scale.data_ptr(), *tail))
        else:
            check(qc.qc_qlinear(*head, L.pw.blob.data_ptr(), L.pw.scale.data_ptr(), *tail))

    def quant_stage(L):
        c = L.case
        head = (L.x.data_ptr(), qc.QC_BF16, c.M, c.K)
        tail = (L.ws.data_ptr(), L.ws.numel(), stream)
        if asym:
            check(qc.qc_qlinear_asym_quant(*head, act_bits, *tail))
        elif rot:
            check(qc.qc_qlinear_quant_rot(*head, act_bits, rot, *tail))
        else:
            check(qc.qc_qlinear_quant_bits(*head, act_bits, *tail))

    def gemm_stage(L):
        c = L.case
        tail = (c.bits, c.N, L.bias.data_ptr(), L.epi, L.Y.data_ptr(), qc.QC_OUT_BF16, stream)
        if asym:
            check(qc.qc_qlinear_asym_gemm(L.ws.data_ptr(), L.ws.numel(), c.M, c.K,
                                          L.pw.blob.data_ptr(), L.pw.scale.data_ptr(),
                                          L.row_sums.data_ptr(), *tail))
        else:
            check(qc.qc_qlinear_gemm(L.ws.data_ptr(), L.ws.numel(), c.M, c.K,
                                     L.pw.blob.data_ptr(), L.pw.scale.data_ptr(), *tail))

    def delta_stage(on=None):
        check(qc.qc_latent_delta(cur.data_ptr(), prev.data_ptr(), n_lat, out3.data_ptr(),
                                 dws.data_ptr(), dws.numel(), stream if on is None else on))

    def pack_stage(L):
        c = L.case
        if rot:
            check(qc.qc_pack_weight_rot(L.W.data_ptr(), c.N, c.K, c.bits, rot,
                                        L.pw.blob.data_ptr(), L.pw.scale.data_ptr(), stream))
        else:
            check(qc.qc_pack_weight(L.W.data_ptr(), c.N, c.K, c.bits, L.pw.blob.data_ptr(),
                                    L.pw.scale.data_ptr(), stream))

    def step():
        for L in layers:
            qlinear(L)
        if not sweep:
            delta_stage(side_stream)

    # ---- headline: K steps between two full synchronisations ----------------------------
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    with PowerSampler() as sampler:
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    device_info = dict(name=torch.cuda.get_device_name(0), **sampler.summary())
    ops = sum(L.ops for L in layers)
    value = ops / (ms_per_step * 1e-3) / 1e12

    # ---- per-kernel durations --------------------------------------------------------------
    if sweep:
        batch, rounds = 1, 3
    else:
        batch = 20
        rounds = max(3, min(steps, 600) // batch)
    for _ in range(min(warmup, 300)):
        step()
    per = {
        "quant": batch_times_us(lambda: [quant_stage(L) for L in layers], batch, rounds),
        "gemm": batch_times_us(lambda: [gemm_stage(L) for L in layers], batch, rounds),
        "pack": batch_times_us(lambda: [pack_stage(L) for L in layers], 1, 5),
    }
    if not sweep:
        per["delta"] = batch_times_us(delta_stage, batch, rounds)
        # The same two kernels on inputs that are cold in the L2s and the 256 MB Infinity Cache:
        # each launch takes the next of enough distinct copies of its input to exceed 320 MB
        # (a layer whose activations are larger than that is cold anyway).
        L0 = layers[0]
        copies = max(2, -(-(320 << 20) // (L0.x.numel() * 2)))
        xs = [L0.x] + [L0.x.clone() for _ in range(copies - 1)]
        turn = [0]

        def quant_cold():
            x = xs[turn[0] % copies]
            turn[0] += 1
            check(qc.qc_qlinear_quant_bits(x.data_ptr(), qc.QC_BF16, L0.case.M, L0.case.K, act_bits,
                                           L0.ws.data_ptr(), L0.ws.numel(), stream)
                  if not (asym or rot) else
                  (qc.qc_qlinear_asym_quant(x.data_ptr(), qc.QC_BF16, L0.case.M, L0.case.K, act_bits,
                                            L0.ws.data_ptr(), L0.ws.numel(), stream) if asym else
                   qc.qc_qlinear_quant_rot(x.data_ptr(), qc.QC_BF16, L0.case.M, L0.case.K, act_bits,
                                           rot, L0.ws.data_ptr(), L0.ws.numel(), stream)))
        per["quant_cold"] = batch_times_us(quant_cold, copies, max(3, 60 // copies))
        pairs = -(-(320 << 20) // (2 * n_lat * 4))
        lat = [(cur, prev)] + [(cur.clone(), prev.clone()) for _ in range(pairs - 1)]

        def delta_cold():
            a, b = lat[turn[0] % pairs]
            turn[0] += 1
            check(qc.qc_latent_delta(a.data_ptr(), b.data_ptr(), n_lat, out3.data_ptr(),
                                     dws.data_ptr(), dws.numel(), stream))
        per["delta_cold"] = batch_times_us(delta_cold, pairs, 6)
        del xs, lat

    if args.calibration_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()

    traffic = MEASURED_TRAFFIC_BYTES.get(args.workload, {}) if args.variant == "a8" else {}
    gemm_us = per["gemm"]["avg_us"]
    gemm_tops = ops / (gemm_us * 1e-6) / 1e12
    quant_bytes = sum(c.M * c.K * 3 + 4 * c.M for c in cases)
    quant_gbs = quant_bytes / (per["quant"]["avg_us"] * 1e-6) / 1e9
    kernel_name = ("gemm_kernel<8|4, bf16, none|gelu_tanh> (112 launches)" if sweep else
                   f"gemm_kernel<{cases[0].bits}, bf16, {cases[0].epi}>")

    result = {
        "metric": "quantized-linear int8 TOPS, whole qc_qlinear" +
                  ("" if sweep else " + qc_latent_delta") + " step, 1 MI355X",
        "value": round(value, 2),
        "unit": "TOPS",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8 (int32 accumulate; bf16 in/out, fp32 scales)",
        "data": "synthetic",
        "config": {"workload": describe, "name": args.workload, "variant": args.variant,
                   "activation_quantizer": {"a8": "symmetric int8 per token", "a6": "symmetric 6 bit per token",
                                            "a4": "symmetric 4 bit per token",
                                            "rot128": "Walsh-Hadamard blocks of 128 columns, then symmetric int8 per token",
                                            "asym": "asymmetric uint8 per token with zero point"}[args.variant],
                   "layers": len(cases),
                   "w4_layers": w4_layers, "M": M, "seed": cases[0].seed,
                   "offline_not_in_step": "qc_pack_weight",
                   "streams": "qc_qlinear on the current stream" +
                              ("" if sweep else ", qc_latent_delta on a second one")},
        "device": device_info,
        "roofline": {"bound": "mfma", "kernel": kernel_name,
                     "achieved": round(gemm_tops, 1), "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                     "frac": round(gemm_tops / PEAK_INT8_TOPS, 4),
                     "traffic": traffic.get("gemm"),
                     "ops_per_launch": ops / len(cases), "launches_per_step": len(cases),
                     "avg_launch_us": round(gemm_us / len(cases), 2)},
        "kernels": {
            "quant_act": {"bound": "hbm", "achieved": round(quant_gbs, 1), "peak": PEAK_HBM_GBS,
                          "unit": "GB/s", "frac": round(quant_gbs / PEAK_HBM_GBS, 4),
                          "bytes_per_launch": quant_bytes / len(cases),
                          "avg_launch_us": round(per["quant"]["avg_us"] / len(cases), 2),
                          "traffic": traffic.get("quant")},
            "pack_weight_offline": {"avg_launch_us": round(per["pack"]["avg_us"] / len(cases), 2)},
            # quantization + GEMM + epilogue of the layer(s), without the latent delta
            "qlinear_whole_call": {
                "achieved": round(ops / ((per["quant"]["avg_us"] + gemm_us) * 1e-6) / 1e12, 1),
                "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                "frac": round(ops / ((per["quant"]["avg_us"] + gemm_us) * 1e-6) / 1e12 / PEAK_INT8_TOPS, 4),
                "avg_us": round((per["quant"]["avg_us"] + gemm_us) / len(cases), 2)},
        },
    }
    if not sweep:
        c = cases[0]
        result["config"].update({"K": c.K, "N": c.N, "weight_bits": c.bits, "epilogue": c.epi})
        delta_bytes = 2 * n_lat * 4 + 12
        delta_gbs = delta_bytes / (per["delta"]["avg_us"] * 1e-6) / 1e9
        result["kernels"]["latent_delta"] = {
            "bound": "hbm", "achieved": round(delta_gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": round(delta_gbs / PEAK_HBM_GBS, 4), "bytes_per_launch": delta_bytes,
            "avg_launch_us": round(per["delta"]["avg_us"], 2),
            "note": "two launches per call; the 33.5 MB of inputs stay resident in the 256 MB "
                    "Infinity Cache between calls (warm)",
            "traffic": traffic.get("delta"),
            "cold": {"avg_launch_us": round(per["delta_cold"]["avg_us"], 2),
                     "achieved": round(delta_bytes / (per["delta_cold"]["avg_us"] * 1e-6) / 1e9, 1),
                     "frac": round(delta_bytes / (per["delta_cold"]["avg_us"] * 1e-6) / 1e9 / PEAK_HBM_GBS, 4)}}
        qc_us = per["quant_cold"]["avg_us"]
        result["kernels"]["quant_act"]["cold"] = {
            "avg_launch_us": round(qc_us, 2), "achieved": round(quant_bytes / (qc_us * 1e-6) / 1e9, 1),
            "frac": round(quant_bytes / (qc_us * 1e-6) / 1e9 / PEAK_HBM_GBS, 4),
            "note": "each launch reads the next of enough distinct input copies to exceed 320 MB"}
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cases[0], act_bits, rot, asym)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
