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
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding.lib()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fbsr_[a-z_0-9]+)\s*\(", text)))


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
                      ("FBSR_RNE", b.RNE), ("FBSR_SRFF", b.SRFF), ("FBSR_SRF", b.SRF), ("FBSR_SRC", b.SRC),
                      ("FBSR_OK", b.OK), ("FBSR_EINVAL", b.EINVAL), ("FBSR_EALIGN", b.EALIGN),
                      ("FBSR_ERANGE", b.ERANGE), ("FBSR_EDEVICE", b.EDEVICE)):
        assert re.search(r"\b%s\s*=\s*%d\b" % (name, val), text), name
    assert re.search(r"#define\s+FBSR_MAX_NBITS\s+%d" % b.MAX_NBITS, text)


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
    for fmt, var, nb in ((3, 1, 2), (-1, 1, 2), (0, 4, 2), (0, -1, 2), (0, 1, 0), (0, 2, 17), (1, 3, -5)):
        assert L.fbsr_round(p(good), p(good), 8, fmt, var, nb, 0, 0, None) == EINVAL
        assert L.fbsr_bias_stats(p(good), None, 8, fmt, var, nb, 0, 0, 4, 0, 2, p(good), p(good), 1 << 20, None) == EINVAL
    assert L.fbsr_sgd_update(p(good), p(good), 8, 0.1, 5, 2, 0, 0, 0, None) == EINVAL
    assert L.fbsr_sgd_update(p(good), p(good), 8, 0.1, 1, 99, 0, 0, 0, None) == EINVAL
    for src, fmt in ((2, 1), (0, 0), (1, 3), (-1, 2)):
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
    need = L.fbsr_bias_stats_workspace_bytes(8, 2)
    assert need > 0
    assert L.fbsr_bias_stats(p(good), None, 8, 0, 1, 2, 0, 0, 4, 0, 2, p(good), p(good), need - 1, None) == ERANGE


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
