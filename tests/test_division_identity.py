"""The fused QAT kernel divides by its two launch-uniform bias corrections with a multiply and two fused
multiply-adds.  That this equals the correctly rounded division is a statement about IEEE binary32 arithmetic,
checked here on the CPU (tests/division_by_uniform_check.c, plain C with fmaf): all bf16 significands of both signs
against every 37th divisor significand at ten exponent pairs, plus zeros, infinities and the range's ends.  CPU only."""
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
