"""The quantised epilogue divides by its two steps with a reciprocal sequence instead of a division per
element; step_quotient_check.c shows on the host, exhaustively over the quotients that decide an integer
code, that the sequence gives the IEEE quotient (what the oracle computes)."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_reciprocal_sequence_equals_ieee_division(tmp_path):
    exe = str(tmp_path / "step_quotient_check")
    subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-o", exe, os.path.join(HERE, "step_quotient_check.c"), "-lm"])
    # the steps of the test and benchmark workloads, and one with a long significand
    r = subprocess.run([exe, "0.031", "0.043", "0.33333334"], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "total mismatches 0" in r.stdout
