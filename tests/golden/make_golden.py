"""Writes tests/golden/oracle_outputs.json: what the CPU oracle computes for small seeded cases.

Run as `python tests/golden/make_golden.py` from the repository root.  It calls only the
oracle and the seeded input generators, never the GPU library, so the stored values are the
oracle's.  The paper (arxiv 2503.06545) prints no worked numeric example of its quantizer or of
Eq. (5), so there is no fixture taken from the paper itself; this file instead freezes the
oracle, so that a later change to its arithmetic shows up as a diff of stored numbers, and
gives the GPU tests expected values that exist before the GPU code runs.

Codes and accumulators are stored as CRC-32 of their bytes plus a few plain samples; scales
as binary32 bit patterns; floating-point results as hexadecimal doubles.
"""
import json
import os
import sys
import zlib

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2503_06545_amd import synth  # noqa: E402

SAMPLES = [(0, 0), (1, 5), (17, 300), (255, 1151), (128, 640)]


def crc(a: np.ndarray) -> int:
    return zlib.crc32(np.ascontiguousarray(a).tobytes()) & 0xFFFFFFFF


def linear_case(case, bits, epi, act_bits=8, rot_block=0, rows=None):
    x = case.x() if rows is None else case.x_rows(0, rows)
    W, b = case.weight(), case.bias()
    if rot_block:
        qw, sw = oracle.quant_weight_rot(W, bits, rot_block)
        r = oracle.qlinear_rot(x, qw, sw, rot_block, b, getattr(oracle, "EPI_" + epi.upper()), act_bits)
    else:
        qw, sw = oracle.quant_weight(W, bits)
        r = oracle.qlinear(x, qw, sw, b, getattr(oracle, "EPI_" + epi.upper()), act_bits)
    M, N = r["y"].shape
    pts = [(m % M, n % N) for m, n in SAMPLES]
    return {
        "case": case.name, "rows": int(M), "bits": bits, "epi": epi, "act_bits": act_bits,
        "rot_block": rot_block,
        "qw_crc32": crc(qw), "sw_crc32": crc(sw), "qx_crc32": crc(r["qx"]), "sx_crc32": crc(r["sx"]),
        "acc_crc32": crc(r["acc"]),
        "sx_bits_first4": [int(v) for v in r["sx"][:4].view(np.uint32)],
        "sw_bits_first4": [int(v) for v in sw[:4].view(np.uint32)],
        "acc_samples": [int(r["acc"][m, n]) for m, n in pts],
        "y_samples_hex": [float(r["y"][m, n]).hex() for m, n in pts],
        "y_sum_hex": float(np.sum(r["y"])).hex(),
    }


def build():
    out = {"linear": [], "reductions": {}}
    out["linear"].append(linear_case(synth.TINY, 8, "none"))
    out["linear"].append(linear_case(synth.TINY, 4, "gelu_tanh"))
    out["linear"].append(linear_case(synth.TINY, 4, "gelu_erf", act_bits=6))
    out["linear"].append(linear_case(synth.TINY, 8, "none", rot_block=128))
    out["linear"].append(linear_case(synth.QKV_256, 8, "none", rows=64))
    cur, prev = synth.latent_pair(seed=3, n=100003)
    out["reductions"]["latent_delta_seed3_n100003_hex"] = [float(v).hex() for v in oracle.latent_delta(cur, prev)]
    out["reductions"]["layer_similarity_seed3_n100003_hex"] = [float(v).hex() for v in oracle.layer_similarity(cur, prev)]
    out["reductions"]["frame_gradient_seed3_7x14286_hex"] = [
        float(v).hex() for v in oracle.frame_gradient(cur[:7 * 14286].reshape(7, 14286))]
    prevs = np.stack([prev, (prev * np.float32(0.5)).astype(np.float32)])
    out["reductions"]["cumulative_variation_seed3_n100003_hex"] = [
        float(v).hex() for v in oracle.cumulative_variation(cur, prevs)]
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_outputs.json")
    with open(path, "w") as f:
        json.dump(build(), f, indent=1, sort_keys=True)
        f.write("\n")
    print("wrote", path)
