"""The quantizer's scale factor (max - min) / (2^b - 1) (App. B "Preliminaries") is computed on the GPU as a
multiplication by the rounded reciprocal plus one exact correction step.  That this equals IEEE division is a fact about
binary32 arithmetic, checked here on the CPU with the C library's fused multiply-add (a sample of the bit patterns in
the test; tests/division_check.c with stride 1 walks all of them)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))


def test_corrected_reciprocal_multiplication_equals_division(tmp_path):
    exe = str(tmp_path / "division_check")
    subprocess.run(["gcc", "-O2", "-ffp-contract=off", "-o", exe, os.path.join(HERE, "division_check.c"), "-lm"], check=True)
    r = subprocess.run([exe, "61"], capture_output=True, text=True)        # a prime stride: all low-bit patterns occur
    assert r.returncode == 0, r.stdout
    assert r.stdout.count("mismatches=0") == 5
