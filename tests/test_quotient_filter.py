"""The quantizer kernel decides its codes with a cheap quotient and falls back to the IEEE
division only near half-integers (csrc/awq_quantize.hip, fast_rint_quotient).  That this gives
rint(fl(n / d)) for every step and every numerator is shown exhaustively by a small C program
(quotient_filter_check.c: every normal binary16 step, the three reciprocals the hardware may
return, every half-integer that matters, every binary32 numerator around it); the same program
built with a band that is too narrow must report misses, so the check has teeth."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "quotient_filter_check.c")


def _build(tmp_path, name, *defs):
    exe = str(tmp_path / name)
    subprocess.run(["gcc", "-O2", "-ffp-contract=off", *defs, "-o", exe, SRC, "-lm"], check=True)
    return exe


def test_band_value_is_the_kernels():
    kernel = open(os.path.join(HERE, "..", "paper_2306_00978_amd", "csrc", "awq_quantize.hip")).read()
    assert "constexpr float AWQ_TIE_BAND = 1.52587890625e-05f;" in kernel
    assert "#define BAND_VALUE 1.52587890625e-05f" in open(SRC).read()


def test_fast_quotient_with_the_band_equals_the_ieee_quotient_everywhere(tmp_path):
    p = subprocess.run([_build(tmp_path, "check")], capture_output=True, text=True, timeout=600)
    assert p.returncode == 0, p.stdout[-2000:]
    assert "misses 0" in p.stdout


def test_a_band_that_is_too_narrow_is_caught(tmp_path):
    p = subprocess.run([_build(tmp_path, "narrow", "-DBAND_VALUE=1e-7f")], capture_output=True, text=True,
                       timeout=600)
    assert p.returncode == 1 and "MISS" in p.stdout
