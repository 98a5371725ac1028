"""Compile libqc.so for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libqc.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["qc_api.hip", "qc_quant.hip", "qc_pack.hip", "qc_gemm.hip", "qc_delta.hip"]
ROOFS = os.path.join(HERE, "qc_roofs")  # stand-alone roofline micro-benchmark

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",                      # the quantizer's binary32 steps are part of the contract
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
    subprocess.run([HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj], check=True)
    return obj


def _compile_roofs(_=None) -> str:
    subprocess.run([HIPCC, *FLAGS, os.path.join(CSRC, "qc_roofs.hip"), "-o", ROOFS], check=True)
    return ROOFS


def build(verbose: bool = True) -> str:
    """Always recompiles every source, relinks libqc.so and rebuilds the qc_roofs program."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES) + 1)) as pool:
        roofs = pool.submit(_compile_roofs)
        objs = list(pool.map(_compile, SOURCES))
        roofs.result()
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB], check=True)
    if verbose:
        print(f"built {LIB}", file=sys.stderr)
    return LIB


if __name__ == "__main__":
    build()
