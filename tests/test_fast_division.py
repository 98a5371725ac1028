"""The activation-quantization kernel replaces the per-element IEEE division by a reciprocal
and one fused residual correction.  This host test shows the replacement is exact where it
matters: identical quotient bits for every quotient that can round to a non-zero code, and
identical int8 codes everywhere (all bf16 inputs x many scales, random binary32 inputs and
constructed near-ties)."""
import os
import subprocess
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))


def test_reciprocal_plus_one_fma_correction_equals_ieee_division():
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "fast_division_check")
        subprocess.run(["gcc", "-O2", "-mfma", "-ffp-contract=off",
                        os.path.join(HERE, "fast_division_check.c"), "-o", exe, "-lm"], check=True)
        for qmax, scales, randoms in (("127", "400", "20000000"), ("31", "150", "6000000"),
                                      ("7", "150", "6000000")):
            out = subprocess.run([exe, scales, randoms, qmax], check=True, capture_output=True,
                                 text=True)
            pairs, bad_quotients, bad_codes = (int(v) for v in out.stdout.split())
            assert pairs > 5_000_000
            assert bad_quotients == 0 and bad_codes == 0, (qmax, bad_quotients, bad_codes)
        # scales whose significand is all ones or nearly: the reciprocal is least accurate there
        out = subprocess.run([exe, "4000", "0", "127", "edge"], check=True, capture_output=True,
                             text=True)
        pairs, bad_quotients, bad_rounded = (int(v) for v in out.stdout.split())
        assert pairs > 8_000_000 and bad_quotients == 0 and bad_rounded == 0
        # the asymmetric quantizer: rows far from zero, quotients far above the code range
        for levels in ("255", "63", "15"):
            out = subprocess.run([exe, "1000000", "24", levels, "asym"], check=True,
                                 capture_output=True, text=True)
            pairs, bad_rounded, bad_codes = (int(v) for v in out.stdout.split())
            assert pairs > 3_000_000
            assert bad_rounded == 0 and bad_codes == 0, (levels, bad_rounded, bad_codes)
