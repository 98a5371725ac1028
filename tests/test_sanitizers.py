"""The CPU oracle and the host-side division check under AddressSanitizer and
UndefinedBehaviorSanitizer: both are plain C, compiled here with gcc's sanitizers and run on a
slice of the cases the pins use (out-of-bounds indexing, signed overflow, bad shifts and
misaligned accesses in the checker would show up here)."""
import os
import shutil
import subprocess
import sys
import textwrap

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


def _asan_runtime():
    out = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    return out if os.path.isabs(out) and os.path.exists(out) else None


@pytest.mark.skipif(shutil.which("gcc") is None or _asan_runtime() is None, reason="gcc with libasan is needed")
def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    lib = tmp_path / "libqc_oracle_san.so"
    subprocess.run(["gcc", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", *SAN,
                    os.path.join(ROOT, "oracle", "qc_oracle.c"), "-o", str(lib), "-lm"], check=True)
    # A fresh interpreter with the sanitizer runtime loaded first; the oracle's Python front is
    # pointed at the instrumented library and runs a slice of every function family.
    script = textwrap.dedent(f"""
        import sys
        import numpy as np
        sys.path.insert(0, {ROOT!r})
        import oracle
        rng = np.random.default_rng(1)
        for M, K, N in ((5, 16, 3), (33, 200, 77), (64, 1152, 130)):
            x = rng.standard_normal((M, K)).astype(np.float32)
            x[0] = 0.0
            W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
            b = (rng.standard_normal(N) * 0.01).astype(np.float32)
            for bits in (8, 4):
                qw, sw = oracle.quant_weight(W, bits)
                for epi in (oracle.EPI_NONE, oracle.EPI_GELU_TANH, oracle.EPI_GELU_ERF):
                    for act_bits in (8, 6, 4):
                        oracle.qlinear(x, qw, sw, b, epi, act_bits)
                oracle.qlinear_asym(x, qw, sw, b, oracle.EPI_NONE, 8)
                if K % 16 == 0:
                    qr, sr = oracle.quant_weight_rot(W, bits, 16)
                    oracle.qlinear_rot(x, qr, sr, 16, b, oracle.EPI_NONE, 8)
        a, c = rng.standard_normal(10003).astype(np.float32), rng.standard_normal(10003).astype(np.float32)
        oracle.latent_delta(a, c)
        oracle.layer_similarity(a, c)
        oracle.frame_gradient(a[:10000].reshape(10, 1000))
        oracle.cumulative_variation(a, [c, a])
        print("oracle ok under sanitizers")
    """)
    # the sanitizer runtime has to be the first preloaded library; whatever is preloaded already stays
    preload = ":".join(p for p in (_asan_runtime(), os.environ.get("LD_PRELOAD", "")) if p)
    env = dict(os.environ, LD_PRELOAD=preload, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0",
               OMP_NUM_THREADS="2", QC_ORACLE_LIB=str(lib))
    r = subprocess.run([sys.executable, "-c", script], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "oracle ok under sanitizers" in r.stdout, (r.stdout[-500:], r.stderr[-3000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-3000:]


@pytest.mark.skipif(shutil.which("gcc") is None or _asan_runtime() is None, reason="gcc with libasan is needed")
def test_fast_division_check_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "fast_division_check_san"
    subprocess.run(["gcc", "-mfma", "-ffp-contract=off", *SAN,
                    os.path.join(ROOT, "tests", "fast_division_check.c"), "-o", str(exe), "-lm"], check=True)
    for args in (["20", "200000", "127"], ["100", "0", "127", "edge"], ["20000", "24", "255", "asym"]):
        r = subprocess.run([str(exe), *args], capture_output=True, text=True, timeout=300,
                           env=dict(os.environ, ASAN_OPTIONS="detect_leaks=0"))
        assert r.returncode == 0, (args, r.stdout[-500:], r.stderr[-3000:])
        assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
        assert all(int(v) == 0 for v in r.stdout.split()[1:]), (args, r.stdout)
