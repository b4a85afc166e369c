"""Host-side checks of the C ABI: the library loads, exports every symbol the header declares,
and rejects bad arguments before launching anything.  No GPU needed (no kernel is launched)."""
import ctypes
import os
import re

import pytest

from conftest import ROOT

HEADER = os.path.join(ROOT, "include", "fbsr.h")


@pytest.fixture(scope="module")
def L():
    from paper_2504_20634_amd import binding, build
    if os.environ.get("FBSR_ABI_LIB"):      # a host-sanitized build of the argument checks (tests/test_sanitizers.py)
        binding.LIB_PATH = os.environ["FBSR_ABI_LIB"]
    elif not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding.lib()


def declared_functions():
    """Every function declared in any header under include/ (the product interface and the measurement aids)."""
    names = set()
    for header in sorted(os.listdir(os.path.dirname(HEADER))):
        if header.endswith(".h"):
            text = open(os.path.join(os.path.dirname(HEADER), header)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(fbsr_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(L):
    names = declared_functions()
    assert {"fbsr_round", "fbsr_round_from16", "fbsr_round_block_scaled", "fbsr_qat_adamw_step", "fbsr_sgd_update", "fbsr_bias_stats", "fbsr_bias_stats_workspace_bytes",
            "fbsr_strerror", "fbsr_version"} <= set(names)
    for name in names:
        assert hasattr(L, name), name
    from paper_2504_20634_amd import binding
    assert set(binding.EXPORTS) == set(names)


def test_enums_match_the_header():
    from paper_2504_20634_amd import binding as b
    text = open(HEADER).read()
    for name, val in (("FBSR_FMT_BF16", b.FMT_BF16), ("FBSR_FMT_E4M3", b.FMT_E4M3), ("FBSR_FMT_E5M2", b.FMT_E5M2),
                      ("FBSR_FMT_BINARY8P4", b.FMT_BINARY8P4),
                      ("FBSR_RNE", b.RNE), ("FBSR_SRFF", b.SRFF), ("FBSR_SRF", b.SRF), ("FBSR_SRC", b.SRC),
                      ("FBSR_OK", b.OK), ("FBSR_EINVAL", b.EINVAL), ("FBSR_EALIGN", b.EALIGN),
                      ("FBSR_ERANGE", b.ERANGE), ("FBSR_EDEVICE", b.EDEVICE)):
        assert re.search(r"\b%s\s*=\s*%d\b" % (name, val), text), name
    assert re.search(r"#define\s+FBSR_MAX_NBITS\s+%d" % b.MAX_NBITS, text)
    assert re.search(r"#define\s+FBSR_MAX_NBITS_ROUND\s+%d" % b.MAX_NBITS_ROUND, text)
    for name, val in (("FBSR_FROM_BF16", b.FROM_BF16), ("FBSR_FROM_FP16", b.FROM_FP16), ("FBSR_FROM_FP32", b.FROM_FP32),
                      ("FBSR_SRC_TIES_ODD", b.SRC_TIES_ODD), ("FBSR_RNO", b.RNO), ("FBSR_RNA", b.RNA)):
        assert re.search(r"#define\s+%s\s+%d\b" % (name, val), text), name


def test_strerror_and_version(L):
    assert L.fbsr_version() >= 100
    seen = {L.fbsr_strerror(s) for s in range(5)}
    assert len(seen) == 5 and all(seen)
    assert L.fbsr_strerror(99)


def test_argument_validation_happens_on_the_host(L):
    OK, EINVAL, EALIGN, ERANGE = 0, 1, 2, 3
    p = ctypes.c_void_p
    good = 0x7F0000001000       # never dereferenced: every call below fails validation or has n == 0
    # n == 0 is a no-op even with null pointers
    assert L.fbsr_round(None, None, 0, 0, 1, 2, 0, 0, None) == OK
    assert L.fbsr_sgd_update(None, None, 0, 0.1, 1, 2, 0, 0, 0, None) == OK
    assert L.fbsr_bias_stats(None, None, 0, 0, 1, 2, 0, 0, 1, 0, 1, None, None, 0, None) == OK
    # bad enums / nbits
    for fmt, var, nb in ((4, 1, 2), (-1, 1, 2), (0, 4, 2), (0, -1, 2), (0, 1, 0), (0, 2, 25), (1, 3, -5)):
        assert L.fbsr_round(p(good), p(good), 8, fmt, var, nb, 0, 0, None) == EINVAL
        assert L.fbsr_bias_stats(p(good), None, 8, fmt, var, nb, 0, 0, 4, 0, 2, p(good), p(good), 1 << 20, None) == EINVAL
    # the fused updates take up to 16 bits, everything else up to 24
    assert L.fbsr_bias_stats(p(good), None, 8, 1, 1, 25, 0, 0, 4, 0, 2, p(good), p(good), 1 << 20, None) == EINVAL
    assert L.fbsr_bias_stats(p(good + 2), None, 8, 1, 1, 24, 0, 0, 4, 0, 2, p(good), p(good), 1 << 20, None) == EALIGN
    assert L.fbsr_round_block_scaled(p(good), p(good), p(good), 8, 1, 1, 25, 0, 0, None) == EINVAL
    assert L.fbsr_round_block_scaled(p(good + 2), p(good), p(good), 8, 1, 1, 24, 0, 0, None) == EALIGN
    assert L.fbsr_sgd_update(p(good), p(good), 8, 0.1, 1, 17, 0, 0, 0, None) == EINVAL
    assert L.fbsr_round_from16(p(good), p(good), 8, 0, 1, 1, 25, 0, 0, None) == EINVAL
    assert L.fbsr_round(p(good + 2), p(good), 8, 1, 1, 24, 0, 0, None) == EALIGN      # 24 passes the nbits check
    assert L.fbsr_round_from16(p(good + 1), p(good), 8, 0, 1, 1, 24, 0, 0, None) == EALIGN
    assert L.fbsr_sgd_update(p(good), p(good), 8, 0.1, 5, 2, 0, 0, 0, None) == EINVAL
    assert L.fbsr_sgd_update(p(good), p(good), 8, 0.1, 1, 99, 0, 0, 0, None) == EINVAL
    for src, fmt in ((2, 1), (0, 0), (1, 4), (-1, 2)):
        assert L.fbsr_round_from16(p(good), p(good), 8, src, fmt, 1, 2, 0, 0, None) == EINVAL
    assert L.fbsr_round_from16(None, None, 0, 0, 1, 1, 2, 0, 0, None) == OK
    assert L.fbsr_round_from16(p(good + 1), p(good), 8, 0, 1, 1, 2, 0, 0, None) == EALIGN
    assert L.fbsr_round_from16(p(good), None, 8, 0, 1, 1, 2, 0, 0, None) == EINVAL
    assert L.fbsr_round_block_scaled(None, None, None, 0, 1, 1, 2, 0, 0, None) == OK
    assert L.fbsr_round_block_scaled(p(good), p(good), p(good), 8, 0, 1, 2, 0, 0, None) == EINVAL      # bf16 elements
    assert L.fbsr_round_block_scaled(p(good), p(good), None, 8, 1, 1, 2, 0, 0, None) == EINVAL
    assert L.fbsr_round_block_scaled(p(good + 2), p(good), p(good), 8, 1, 1, 2, 0, 0, None) == EALIGN
    hp = (ctypes.c_float * 7)(1e-3, 0.9, 0.999, 1e-8, 0.0, 0.1, 0.001)
    assert L.fbsr_qat_adamw_step(None, None, None, None, 0, 1, hp, 1, 3, 0, 0, 0, None) == OK
    assert L.fbsr_qat_adamw_step(p(good), p(good), p(good), p(good), 8, 0, hp, 1, 3, 0, 0, 0, None) == EINVAL   # bf16 target
    assert L.fbsr_qat_adamw_step(p(good), p(good), p(good), p(good), 8, 1, None, 1, 3, 0, 0, 0, None) == EINVAL
    assert L.fbsr_qat_adamw_step(p(good), None, p(good), p(good), 8, 1, hp, 1, 3, 0, 0, 0, None) == EINVAL
    assert L.fbsr_qat_adamw_step(p(good), p(good), p(good + 1), p(good), 8, 1, hp, 1, 3, 0, 0, 0, None) == EALIGN
    assert L.fbsr_qat_adamw_step(p(good), p(good), p(good), p(good), 8, 1, hp, 1, 17, 0, 0, 0, None) == EINVAL
    # RNE ignores nbits
    assert L.fbsr_round(None, p(good), 8, 0, 0, 99, 0, 0, None) == EINVAL      # (null x, not nbits)
    # null pointers with n > 0
    assert L.fbsr_round(None, p(good), 8, 0, 1, 2, 0, 0, None) == EINVAL
    assert L.fbsr_round(p(good), None, 8, 0, 1, 2, 0, 0, None) == EINVAL
    assert L.fbsr_sgd_update(None, p(good), 8, 0.1, 1, 2, 0, 0, 0, None) == EINVAL
    assert L.fbsr_bias_stats(p(good), None, 8, 0, 1, 2, 0, 0, 4, 0, 2, None, p(good), 1 << 20, None) == EINVAL
    assert L.fbsr_bias_stats(p(good), None, 8, 0, 1, 2, 0, 0, 4, 0, 2, p(good), None, 1 << 20, None) == EINVAL
    # misaligned pointers
    assert L.fbsr_round(p(good + 2), p(good), 8, 0, 1, 2, 0, 0, None) == EALIGN
    assert L.fbsr_round(p(good), p(good + 1), 8, 0, 1, 2, 0, 0, None) == EALIGN       # bf16 codes need 2
    assert L.fbsr_sgd_update(p(good + 1), p(good), 8, 0.1, 1, 2, 0, 0, 0, None) == EALIGN
    assert L.fbsr_bias_stats(p(good), None, 8, 0, 1, 2, 0, 0, 4, 0, 2, p(good + 4), p(good), 1 << 20, None) == EALIGN
    # overflow of the index range, absurd sizes
    assert L.fbsr_round(p(good), p(good), 8, 0, 1, 2, 0, (1 << 64) - 4, None) == EINVAL
    assert L.fbsr_round(p(good), p(good), (1 << 38) + 1, 0, 1, 2, 0, 0, None) == EINVAL
    # statistics: group 0, bins out of range, workspace too small
    assert L.fbsr_bias_stats(p(good), None, 8, 0, 1, 2, 0, 0, 0, 0, 2, p(good), p(good), 1 << 20, None) == EINVAL
    assert L.fbsr_bias_stats(p(good), None, 8, 0, 1, 2, 0, 0, 4, 0, 1, p(good), p(good), 1 << 20, None) == ERANGE
    assert L.fbsr_bias_stats(p(good), None, 8, 0, 1, 2, 0, 0, 4, 1, 4, p(good), p(good), 1 << 20, None) == ERANGE
    # generic formats of up to 16 bits
    b16 = (ctypes.c_int32 * 8)(16, 11, 15, 0x7BFF, 0x7C00, 0x7E00, 1, 1)
    assert L.fbsr_format16_check(b16) == OK and L.fbsr_format8_check(b16) == EINVAL
    assert L.fbsr_format16_check((ctypes.c_int32 * 8)(16, 7, 15, 0x7BFF, -1, -1, 0, 1)) == EINVAL      # P < K - 8
    assert L.fbsr_format16_check((ctypes.c_int32 * 8)(17, 11, 15, 0x7BFF, -1, -1, 0, 1)) == EINVAL
    assert L.fbsr_format16_check(None) == EINVAL
    assert L.fbsr_round_format16(None, 2, None, 0, b16, 1, 3, 0, 0, None) == OK
    assert L.fbsr_round_format16(p(good), 2, p(good), 8, b16, 1, 15, 0, 0, None) == EINVAL      # nbits <= 30 - K
    assert L.fbsr_round_format16(p(good), 3, p(good), 8, b16, 1, 3, 0, 0, None) == EINVAL
    assert L.fbsr_round_format16(p(good), 2, p(good + 1), 8, b16, 1, 3, 0, 0, None) == EALIGN
    assert L.fbsr_round_format16(p(good + 2), 2, p(good), 8, b16, 1, 3, 0, 0, None) == EALIGN
    assert L.fbsr_round_format16(p(good), 2, None, 8, b16, 1, 3, 0, 0, None) == EINVAL
    assert L.fbsr_round_format8(p(good), 2, p(good), 8, b16, 1, 3, 0, 0, None) == EINVAL
    # the entry point with the built-in workspace: same checks, and a size limit of its own
    assert L.fbsr_bias_stats_static(None, None, 0, 0, 1, 2, 0, 0, 1, 0, 1, None, None) == OK
    assert L.fbsr_bias_stats_static(p(good), None, 8, 0, 1, 2, 0, 0, 0, 0, 2, p(good), None) == EINVAL
    assert L.fbsr_bias_stats_static(p(good), None, 8, 0, 1, 2, 0, 0, 4, 0, 1, p(good), None) == ERANGE
    assert L.fbsr_bias_stats_static(p(good), None, 8, 0, 1, 2, 0, 0, 4, 0, 2, p(good + 4), None) == EALIGN
    assert L.fbsr_bias_stats_static(p(good), None, (1 << 28) + 1, 1, 1, 2, 0, 0, 1 << 20, 0, 1024, p(good), None) == ERANGE
    need = L.fbsr_bias_stats_workspace_bytes(8, 2)
    assert need > 0
    assert L.fbsr_bias_stats(p(good), None, 8, 0, 1, 2, 0, 0, 4, 0, 2, p(good), p(good), need - 1, None) == ERANGE


def test_named_formats_and_descriptor_checks(L):
    """Host-only entry points: the named descriptors equal the ones the oracle's pins were written with
    (tests/test_oracle_format8.py states them from the formats' public definitions), and both sides accept and
    reject the same descriptors."""
    import test_oracle_format8 as pins
    from oracle import fbsr_oracle
    from paper_2504_20634_amd import binding as b
    names = {"ocp_e4m3": pins.E4M3, "ocp_e5m2": pins.E5M2, "ocp_e3m2": pins.E3M2, "ocp_e2m3": pins.E2M3, "ocp_e2m1": pins.E2M1}
    names.update({"p3109_binary8p%d" % P: pins.p3109(P) for P in range(1, 8)})
    for name, want in names.items():
        assert b.format8_named(name).astuple() == tuple(want), name
        assert b.format8_check(want)
    for bad in ("", "ocp_e4m3 ", "p3109_binary8p0", "p3109_binary8p8", "p3109_binary8p44", "bf16"):
        with pytest.raises(b.FbsrError):
            b.format8_named(bad)
    assert L.fbsr_format8_named(None, None) == 1 and L.fbsr_format8_check(None) == 1
    # a sweep of descriptors, valid and not: the library and the oracle agree on every one
    import itertools
    checked = 0
    for K, P, B, mx, inf, nan, ns, nz in itertools.product((1, 2, 4, 8, 9), (0, 1, 3, 7, 8), (-1, 0, 7, 96, 97),
                                                           (0, 3, 7, 0x7B, 0x7E, 0x7F, 0x80), (-1, 0x7C, 0x7F),
                                                           (-1, 0x7E, 0x7F, 0x80, 0xFF, 0x100), (0, 1), (0, 1)):
        d = (K, P, B, mx, inf, nan, ns, nz)
        assert b.format8_check(d) == fbsr_oracle.format8_check(d), d
        checked += 1
    assert checked > 10000


def test_format8_argument_validation(L):
    from paper_2504_20634_amd import binding as b
    OK, EINVAL, EALIGN = 0, 1, 2
    p = ctypes.c_void_p
    good = 0x7F0000001000
    f = b.format8_named("p3109_binary8p4")
    ref = ctypes.byref(f)
    assert L.fbsr_round_format8(None, 2, None, 0, ref, 1, 3, 0, 0, None) == OK
    assert L.fbsr_round_format8(p(good), 2, p(good), 8, None, 1, 3, 0, 0, None) == EINVAL
    for src, var, nb in ((3, 1, 3), (-1, 1, 3), (2, 7, 3), (2, -1, 3), (2, 1, 0), (2, 4, 25), (2, 3, -2)):
        assert L.fbsr_round_format8(p(good), src, p(good), 8, ref, var, nb, 0, 0, None) == EINVAL
    bad = b.Format8(8, 4, 8, 0x7E, 0x7E, 0x80, 0, 0)
    assert L.fbsr_round_format8(p(good), 2, p(good), 8, ctypes.byref(bad), 1, 3, 0, 0, None) == EINVAL
    assert L.fbsr_round_format8(None, 2, p(good), 8, ref, 1, 3, 0, 0, None) == EINVAL
    assert L.fbsr_round_format8(p(good), 2, None, 8, ref, 1, 3, 0, 0, None) == EINVAL
    assert L.fbsr_round_format8(p(good + 2), 2, p(good), 8, ref, 1, 3, 0, 0, None) == EALIGN
    assert L.fbsr_round_format8(p(good + 2), 2, p(good), 8, ref, 4, 24, 0, 0, None) == EALIGN      # 24 passes the nbits check
    assert L.fbsr_round_format8(p(good + 1), 0, p(good), 8, ref, 1, 3, 0, 0, None) == EALIGN
    assert L.fbsr_round_format8(p(good), 2, p(good), (1 << 38) + 1, ref, 1, 3, 0, 0, None) == EINVAL
    assert L.fbsr_round_format8(p(good), 2, p(good), 8, ref, 1, 3, 0, (1 << 64) - 4, None) == EINVAL


def test_qat_format8_argument_validation(L):
    from paper_2504_20634_amd import binding as b
    OK, EINVAL, EALIGN = 0, 1, 2
    p = ctypes.c_void_p
    good = 0x7F0000001000
    f = b.format8_named("p3109_binary8p4")
    ref = ctypes.byref(f)
    hp = (ctypes.c_float * 7)(1e-3, 0.9, 0.999, 1e-8, 0.0, 0.1, 0.001)
    assert L.fbsr_qat_adamw_step_format8(None, None, None, None, 0, ref, hp, 1, 3, 0, 0, 0, None) == OK
    assert L.fbsr_qat_adamw_step_format8(p(good), p(good), p(good), p(good), 8, None, hp, 1, 3, 0, 0, 0, None) == EINVAL
    assert L.fbsr_qat_adamw_step_format8(p(good), p(good), p(good), p(good), 8, ref, None, 1, 3, 0, 0, 0, None) == EINVAL
    assert L.fbsr_qat_adamw_step_format8(p(good), None, p(good), p(good), 8, ref, hp, 1, 3, 0, 0, 0, None) == EINVAL
    assert L.fbsr_qat_adamw_step_format8(p(good), p(good), p(good), p(good + 1), 8, ref, hp, 1, 3, 0, 0, 0, None) == EALIGN
    for var, nb in ((7, 3), (-1, 3), (4, 17), (2, 0)):
        assert L.fbsr_qat_adamw_step_format8(p(good), p(good), p(good), p(good), 8, ref, hp, var, nb, 0, 0, 0, None) == EINVAL
    bad = b.Format8(8, 4, 8, 0x7E, 0x7E, 0x80, 0, 0)
    assert L.fbsr_qat_adamw_step_format8(p(good), p(good), p(good), p(good), 8, ctypes.byref(bad), hp, 1, 3, 0, 0, 0, None) == EINVAL


def test_workspace_size_grows_with_n(L):
    a = L.fbsr_bias_stats_workspace_bytes(1 << 20, 16)
    b = L.fbsr_bias_stats_workspace_bytes(1 << 30, 4096)
    assert 0 < a < b <= (1 << 30) // 16


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    from paper_2504_20634_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libfbsr.so"))
    with pytest.raises(OSError):
        binding.lib()
