"""The fused QAT kernel divides by its two launch-uniform bias corrections with a multiply and two fused
multiply-adds.  That this equals the correctly rounded division is a statement about IEEE binary32 arithmetic,
checked here on the CPU (tests/division_by_uniform_check.c, plain C with fmaf): all bf16 significands of both signs
against every 37th divisor significand at ten exponent pairs, plus zeros, infinities and the range's ends.  Its square
root on that path is the hardware approximation moved to a neighbour by the sign of two residuals, without the usual
rescaling of small inputs: checked the same way (tests/sqrt_correction_check.c) for every significand at ten exponents
from 2^-96 up, from every starting value within one ulp of the root.  Its last division, m / (sqrt(v) + eps), is the full division
sequence without operand scaling (tests/unscaled_division_check.c: every reciprocal start within one ulp), and the root
of the corrected second moment comes from two tables (tests/tabulated_root_check.c: every bf16 code against several
hundred correction values).  CPU only; tests/test_gpu_qat.py runs the kernel's own device functions on the same
operands."""
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


def test_division_without_operand_scaling_is_the_correctly_rounded_quotient(tmp_path):
    exe = tmp_path / "unscaled_division_check"
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-o", str(exe),
                           os.path.join(ROOT, "tests", "unscaled_division_check.c"), "-lm"])
    out = subprocess.run([str(exe), "20000000"], stdout=subprocess.PIPE, check=False)
    bad, corner, cases = (int(v) for v in out.stdout.split())
    assert out.returncode == 0 and bad == 0 and cases > 3e7
    assert corner > 0, "the documented exception (all-ones divisor, start below the rounded reciprocal) was never drawn"


def test_tabulated_root_of_the_corrected_second_moment(tmp_path):
    exe = tmp_path / "tabulated_root_check"
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-o", str(exe),
                           os.path.join(ROOT, "tests", "tabulated_root_check.c"), "-lm"])
    out = subprocess.run([str(exe), "300"], stdout=subprocess.PIPE, check=False)
    bad, cases = (int(v) for v in out.stdout.split())
    assert out.returncode == 0 and bad == 0 and cases == 300 * 32768
