"""The fused kernel's shared-reciprocal division equals the true division (CPU check).

tests/shared_reciprocal_division.c states the sequence and the claim; stride 1 is
the complete check over all 2^32 numerators (run once by hand: no mismatch for any
count 1..64).  Here: every count, every 251st bit pattern (which visits every
exponent, subnormals, infinities and NaNs included), plus the complete check for
the count 6, where the unguarded sequence does fail on subnormal quotients.
"""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
def test_guarded_shared_reciprocal_division_is_exact(tmp_path):
    exe = tmp_path / "shared_reciprocal_division"
    subprocess.check_call(["gcc", "-O2", "-mfma", "-ffp-contract=off", "-fopenmp",
                           os.path.join(HERE, "shared_reciprocal_division.c"), "-o", str(exe), "-lm"])
    out = subprocess.run([str(exe), "1", "64", "251"], capture_output=True, text=True, timeout=600)
    assert out.returncode == 0, out.stdout
    assert "mismatches: 0" in out.stdout
    for k in ("6",):
        out = subprocess.run([str(exe), k, k, "1"], capture_output=True, text=True, timeout=600)
        assert out.returncode == 0, out.stdout
