"""The kernels quantise with x / s computed from the scale's rounded reciprocal and two corrected steps
(no per-element division).  That this reproduces the IEEE quotient bit for bit is a claim about floating
point arithmetic, checked here on the host by a small C program of its own (no kernel, no oracle code):
exhaustively over every significand of x for 96 scales, and on 5e7 random pairs."""
import os
import subprocess
import tempfile


def test_corrected_reciprocal_quotient_equals_ieee_division():
    src = os.path.join(os.path.dirname(os.path.abspath(__file__)), "quotient_check.c")
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "quotient_check")
        base = ["gcc", "-O2", "-ffp-contract=off", "-std=c11", "-o", exe, src, "-lm"]
        # with the host's own fused multiply-add when it has one (fmaf() is exact either way, only slower)
        if subprocess.run(base[:2] + ["-march=native"] + base[2:], capture_output=True).returncode != 0:
            subprocess.run(base, check=True)
        out = subprocess.run([exe, "96", "50000000"], check=False, capture_output=True, text=True, timeout=300)
    assert out.returncode == 0 and out.stdout.strip() == "mismatches 0", out.stdout + out.stderr
