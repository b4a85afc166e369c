"""The fused QAT kernel divides by its two launch-uniform bias corrections with a multiply and two fused
multiply-adds.  That this equals the correctly rounded division is a statement about IEEE binary32 arithmetic,
checked here on the CPU (tests/division_by_uniform_check.c, plain C with fmaf): all bf16 significands of both signs
against every 37th divisor significand at ten exponent pairs, plus zeros, infinities and the range's ends.  Its square
root on that path is the hardware approximation moved to a neighbour by the sign of two residuals, without the usual
rescaling of small inputs: checked the same way (tests/sqrt_correction_check.c) for every significand at ten exponents
from 2^-96 up, from every starting value within one ulp of the root.  CPU only."""
import os
import subprocess

from conftest import ROOT


def test_short_division_is_the_correctly_rounded_quotient(tmp_path):
    exe = tmp_path / "division_check"
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-o", str(exe),
                           os.path.join(ROOT, "tests", "division_by_uniform_check.c"), "-lm"])
    out = subprocess.run([str(exe), "37"], stdout=subprocess.PIPE, check=False)
    bad, cases = (int(v) for v in out.stdout.split())
    assert out.returncode == 0 and bad == 0 and cases > 5e8


def test_sqrt_correction_gives_the_correctly_rounded_root(tmp_path):
    exe = tmp_path / "sqrt_check"
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-o", str(exe),
                           os.path.join(ROOT, "tests", "sqrt_correction_check.c"), "-lm"])
    out = subprocess.run([str(exe), "1"], stdout=subprocess.PIPE, check=False)
    bad, cases = (int(v) for v in out.stdout.split())
    assert out.returncode == 0 and bad == 0 and cases > 1.6e8
