"""Compile libqc.so for gfx950 with hipcc (cross-compiles without a GPU).

Also builds bench/qc_roofs, the stand-alone roofline micro-benchmark bench.py runs beside the
library (it is not part of libqc), and checks the compiler's resource report of every kernel:
the GEMM keeps operand loads in flight across hand-counted waits, which is only right while its
operand registers are never spilled, so a kernel that needs scratch memory fails the build.
"""
from __future__ import annotations

import json
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libqc.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["qc_api.hip", "qc_quant.hip", "qc_pack.hip", "qc_gemm.hip", "qc_delta.hip"]
ROOFS_SRC = os.path.join(ROOT, "bench", "qc_roofs.hip")
ROOFS = os.path.join(ROOT, "bench", "qc_roofs")  # stand-alone roofline micro-benchmark
RESOURCE_REPORT = os.path.join(OBJ_DIR, "kernel_resources.txt")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",                      # the quantizer's binary32 steps are part of the contract
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def _resources(remarks: str):
    """(kernel, vgprs, scratch bytes per lane, waves per SIMD) from the compiler's remarks."""
    out = []
    for block in re.split(r"remark: [^\n]*Function Name: ", remarks)[1:]:
        def num(key):
            m = re.search(key + r": (\d+)", block)
            return int(m.group(1)) if m else -1
        out.append((block.split("\n")[0].split(" [")[0].strip(), num("VGPRs"),
                    num(r"ScratchSize \[bytes/lane\]"), num(r"Occupancy \[waves/SIMD\]")))
    return out


def _compile(src: str):
    obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
    r = subprocess.run([HIPCC, *FLAGS, "-Rpass-analysis=kernel-resource-usage", "-c",
                        os.path.join(CSRC, src), "-o", obj], stderr=subprocess.PIPE, text=True)
    # everything but the resource remarks (with their source excerpts) and the host pass's
    # harmless complaint about the device-only feature flag
    other, keep = [], True
    for line in r.stderr.splitlines():
        if "packed-fp32-ops" in line:
            continue
        if re.search(r"(remark|warning|error|note): ", line) or re.match(r"\d+ (warning|error)s? generated", line):
            keep = "remark: " not in line and "packed-fp32-ops" not in line and " generated" not in line
        if keep and line.strip():
            other.append(line)
    if r.returncode != 0:
        sys.stderr.write(r.stderr)
        raise subprocess.CalledProcessError(r.returncode, r.args)
    if other:
        sys.stderr.write("\n".join(other) + "\n")
    return obj, [(src,) + k for k in _resources(r.stderr)]


def _compile_roofs(_=None) -> str:
    subprocess.run([HIPCC, *FLAGS, ROOFS_SRC, "-o", ROOFS], check=True, stderr=subprocess.DEVNULL)
    return ROOFS


def build(verbose: bool = True) -> str:
    """Always recompiles every source, relinks libqc.so and rebuilds the qc_roofs program."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES) + 1)) as pool:
        roofs = pool.submit(_compile_roofs)
        results = list(pool.map(_compile, SOURCES))
        roofs.result()
    objs = [o for o, _ in results]
    kernels = [k for _, ks in results for k in ks]
    with open(RESOURCE_REPORT, "w") as f:
        for src, name, vgprs, scratch, waves in kernels:
            f.write(f"{src} {name} vgprs={vgprs} scratch_bytes_per_lane={scratch} waves_per_simd={waves}\n")
    spilled = [k for k in kernels if k[3] != 0]
    if not kernels or spilled:
        raise RuntimeError("kernels that use scratch memory (register spills), or no resource "
                           f"report at all: {spilled}")
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB], check=True)
    # which sources the library was built from: the tree travels to the GPU machine without its
    # history, so the benchmark reads the commit from this stamp
    git = subprocess.run(["git", "-C", ROOT, "describe", "--always", "--dirty", "--abbrev=12"],
                         capture_output=True, text=True)
    with open(os.path.join(OBJ_DIR, "build_info.json"), "w") as f:
        json.dump({"git": git.stdout.strip() or None}, f)
    if verbose:
        print(f"built {LIB} ({len(kernels)} kernels, none uses scratch memory)", file=sys.stderr)
    return LIB


if __name__ == "__main__":
    build()
