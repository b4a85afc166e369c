"""Host-only sanitizer runs (AddressSanitizer + UndefinedBehaviorSanitizer; CPU only, no GPU code is instrumented):
the oracle's pins against a sanitized build of the oracle, and the C ABI's host-side argument checks against a
sanitized build of csrc/fbsr_api.hip linked with stand-in launchers that launch nothing."""
import os
import subprocess
import sys

from conftest import ROOT


def _sanitizer_env(**extra):
    runtimes = [subprocess.check_output(["gcc", "-print-file-name=" + n], text=True).strip() for n in ("libasan.so", "libubsan.so")]
    preload = ":".join(runtimes + ([os.environ["LD_PRELOAD"]] if os.environ.get("LD_PRELOAD") else []))
    return dict(os.environ, LD_PRELOAD=preload, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0",
                UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", **extra)


def _clean(run):
    text = run.stdout.decode(errors="replace")
    assert run.returncode == 0, text[-3000:]
    assert "AddressSanitizer" not in text and "runtime error:" not in text, text[-3000:]
    assert " passed" in text


def test_oracle_pins_under_address_and_undefined_sanitizers(tmp_path):
    lib = tmp_path / "liboracle_san.so"
    subprocess.check_call(["g++", "-O1", "-g", "-std=c++17", "-ffp-contract=off", "-fPIC", "-shared", "-pthread",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-o", str(lib),
                           os.path.join(ROOT, "oracle", "fbsr_oracle.cpp")])
    # the pins that sweep 2^20 and more inputs are left to the plain build; every oracle entry point is still reached
    run = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                          os.path.join(ROOT, "tests", "test_oracle_format8.py"), "-x", "-q", "-p", "no:cacheprovider",
                          "-k", "not closed_form and not fig1 and not exact_floor"],
                         env=_sanitizer_env(FBSR_ORACLE_LIB=str(lib)), cwd=ROOT, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    _clean(run)


def test_abi_argument_checks_under_address_and_undefined_sanitizers(tmp_path):
    lib = tmp_path / "libfbsr_hostsan.so"
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.check_call([hipcc, "--cuda-host-only", "-O1", "-g", "-std=c++17", "-fPIC", "-shared",
                           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Wno-unused-command-line-argument",
                           os.path.join(ROOT, "paper_2504_20634_amd", "csrc", "fbsr_api.hip"),
                           os.path.join(ROOT, "tests", "abi_stub_launchers.hip"), "-o", str(lib)],
                          stderr=subprocess.STDOUT)
    run = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_abi.py"), "-x", "-q",
                          "-p", "no:cacheprovider"],
                         env=_sanitizer_env(FBSR_ABI_LIB=str(lib)), cwd=ROOT, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    _clean(run)
