"""Pins for the oracle's generic-format path at widths above 8 bits (any (K, P, B; M) of Sec. II, Eq. (1) with
K <= 16; IEEE binary16 among them): the library's own float16 for decoding and for round-to-nearest-even, exact
rational value tables for other 16-bit formats, counting arguments for the stochastic predicates and the closed-form
biases of Sec. III-E with D = 13 excess bits.  Nothing here touches the GPU library.  CPU only."""
from fractions import Fraction

import numpy as np
import pytest

from exact_model import f32_fraction
from test_oracle_format8 import DRAWING, FROM_BF16, FROM_FP16, FROM_FP32, RNE, SRC, SRC_ODD, SRF, SRFF, TA, TNO, position, ups, value_of

# IEEE 754 binary16: K = 16, P = 11, B = 15, M = 65504 (code 0x7BFF), infinity 0x7C00, quiet NaN 0x7E00 with a sign, -0.
BINARY16 = (16, 11, 15, 0x7BFF, 0x7C00, 0x7E00, 1, 1)
# two further 16-bit layouts, IEEE-like at the top: 6 exponent bits / P = 10, and bf16's layout (P = 8, B = 127) cut one
# binade short, so that M + ulp(M) is still a finite fp32 value (bf16's own M + ulp(M) is 2^128)
E6M9 = (16, 10, 31, (62 << 9) | 0x1FF, 63 << 9, (63 << 9) | 0x100, 1, 1)
E8M7_LOW = (16, 8, 127, (253 << 7) | 0x7F, 254 << 7, (254 << 7) | 0x40, 1, 1)
# a 12-bit format without infinity or NaN (saturating), and a 9-bit one
E5M6_SAT = (12, 7, 15, (31 << 6) | 0x3F, -1, -1, 0, 1)
WIDE = {"binary16": BINARY16, "e6m9": E6M9, "e8m7_low": E8M7_LOW, "e5m6_sat": E5M6_SAT}


def test_width_limits(oracle):
    assert oracle.format16_check(BINARY16) and not oracle.format8_check(BINARY16)
    for d in WIDE.values():
        assert oracle.format16_check(d)
    assert not oracle.format16_check((17, 11, 15, 0x7BFF, 0x7C00, 0x7E00, 1, 1))
    assert not oracle.format16_check((16, 16, 15, 0x7BFF, 0x7C00, 0x7E00, 1, 1))
    assert not oracle.format16_check((16, 11, 15, 0x7BFF, 0x7BFF, 0x7E00, 1, 1))      # infinity not above M
    assert oracle.format16_check((8, 4, 7, 0x7E, -1, 0x7F, 1, 1))                      # narrower formats are fine too


def test_binary16_decodes_like_the_library(oracle):
    codes = np.arange(1 << 16, dtype=np.uint16)
    lib = codes.view(np.float16).astype(np.float64)
    got = np.array([oracle.decode_format16(int(c), BINARY16) for c in codes])
    nan = np.isnan(lib)
    # the descriptor names one NaN code; the other NaN encodings of binary16 are "unused" to it and decode to NaN as well
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], lib[~nan]) and np.array_equal(np.signbit(got[~nan]), np.signbit(lib[~nan]))


@pytest.mark.parametrize("name", ["e6m9", "e8m7_low", "e5m6_sat"])
def test_decode_is_eq1(oracle, name):
    d = WIDE[name]
    K = d[0]
    rng = np.random.default_rng(1)
    for mag in list(rng.integers(0, d[3] + 1, 3000)) + [0, 1, d[3], (1 << (d[1] - 1)) - 1, 1 << (d[1] - 1)]:
        mag = int(mag)
        assert Fraction(oracle.decode_format16(mag, d)) == value_of(mag, d)
        assert Fraction(oracle.decode_format16(mag | (1 << (K - 1)), d)) == -value_of(mag, d)


def test_nearest_even_to_binary16_is_the_library_cast(oracle):
    """fp32 -> binary16, ties to even: numpy's own conversion, over the normal range, the subnormal range, values
    below the smallest subnormal, exact ties, the overflow threshold 65520 and infinities."""
    rng = np.random.default_rng(2)
    field = rng.integers(127 - 30, 127 + 17, 60000, dtype=np.uint32)
    bits = (rng.integers(0, 1 << 32, 60000, dtype=np.uint32) & np.uint32(0x807FFFFF)) | (field << np.uint32(23))
    bits[::5] &= np.uint32(0xFFFFF000)      # many exact ties and representable values
    bits[::7] &= np.uint32(0xFFFFE000)
    x = np.concatenate([bits.view(np.float32), np.array([0.0, -0.0, 65504.0, 65519.99, 65520.0, -65520.0, 65536.0, 1e30, np.inf,
                                                         -np.inf, 2.0 ** -24, 2.0 ** -25, -2.0 ** -25, 2.0 ** -25 * 1.0000001,
                                                         2.0 ** -26, 6.1e-5, 6.0975e-5], dtype=np.float32)])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    got = oracle.round_format16(x, FROM_FP32, BINARY16, RNE, 0, seed=0)
    assert np.array_equal(got, want), np.flatnonzero(got != want)[:10]
    nan = oracle.round_format16(np.array([np.nan, -np.nan], np.float32), FROM_FP32, BINARY16, RNE, 0, seed=0)
    assert nan[0] == 0x7E00 and nan[1] in (0x7E00, 0xFE00)


def test_binary16_source_to_binary16_is_the_identity(oracle):
    codes = np.arange(1 << 16, dtype=np.uint16)
    finite = np.isfinite(codes.view(np.float16).astype(np.float32))
    for variant, nbits in ((RNE, 0), (SRFF, 3), (SRF, 2), (SRC, 5), (SRC_ODD, 4), (TNO, 0), (TA, 0)):
        got = oracle.round_format16(codes, FROM_FP16, BINARY16, variant, nbits, seed=9)
        assert np.array_equal(got[finite], codes[finite]), variant


@pytest.mark.parametrize("name", sorted(WIDE))
@pytest.mark.parametrize("variant", DRAWING)
def test_exhaustive_round_up_counts(oracle, name, variant):
    """Over all 2^N draws, the number that round away from zero equals the counting argument of the predicate
    (Sec. II-B, Eq. (7)) applied to the exact position of |x| between its neighbours from Eq. (1)."""
    d = WIDE[name]
    K, P, B, max_code = d[:4]
    rng = np.random.default_rng(5)
    M = float(value_of(max_code, d))
    lo_exp, hi_exp = 1 - B - (P - 1) - 2, (max_code >> (P - 1)) - B
    xs = (rng.uniform(1.0, 2.0, 60) * 2.0 ** rng.integers(max(lo_exp, -140), min(hi_exp, 120) + 1, 60)).astype(np.float32)
    xs = xs[np.abs(xs.astype(np.float64)) <= M]
    for N in (1, 2, 3, 5):
        for x in xs[:25]:
            a = abs(f32_fraction(x))
            lo, delta = position(a, d)
            count = sum(1 for n in range(1 << N) if (oracle.round_format16_with_n(x, d, variant, N, n) & ((1 << (K - 1)) - 1)) != lo)
            assert count == ups(delta, variant, N), (name, variant, N, float(x), lo, delta)


@pytest.mark.parametrize("N", [1, 2, 3, 4, 13, 14])
def test_fp32_to_binary16_closed_form_biases(oracle, N):
    """Sec. III-E for fp32 -> precision 11 (D = 13 excess bits).  N <= 4: every 16th fp32 input between two neighbours
    (a lattice of 2^-9 ulp, so D = 9 in the closed forms) times all 2^N draws gives exactly SRFF (2^-9 - 2^-N) / 2,
    SRF 2^-10, SRC 0.  N >= 13 = D: every variant is exact SR, P(up) = delta for single inputs (App. A-C)."""
    D = 13
    base = int(np.float32(1.5).view(np.uint32))
    lo = int(np.float32(1.5).astype(np.float16).view(np.uint16))
    xs = (np.uint32(base) + np.arange(1 << D, dtype=np.uint32)).view(np.float32)      # every fp32 in one binary16 interval
    delta_of = lambda x: Fraction(int(np.float32(x).view(np.uint32)) - base, 1 << D)
    ups_of = lambda x, variant: sum(1 for n in range(1 << N) if oracle.round_format16_with_n(x, BINARY16, variant, N, n) != lo)
    if N >= D:
        for x in xs[[1, 2, 77, 4095, 4096, 8191]]:
            for variant in (SRFF, SRF, SRC):
                assert Fraction(ups_of(x, variant), 1 << N) == delta_of(x), (variant, N, float(x))
        return
    stride = xs[::16]
    bias = {v: sum(Fraction(ups_of(x, v), 1 << N) - delta_of(x) for x in stride) / len(stride) for v in (SRFF, SRF, SRC)}
    assert bias[SRFF] == (Fraction(1, 1 << 9) - Fraction(1, 1 << N)) / 2
    assert bias[SRF] == Fraction(1, 1 << 10)
    assert bias[SRC] == 0


def test_overflow_and_specials(oracle):
    """Above M: nearest even on the unbounded grid for a format with an infinity (binary16: 65520 is the tie and M's
    significand is odd, so the tie goes to infinity), saturation without one; NaN keeps its sign where the descriptor
    says so; a format without NaN sends NaN to +-M."""
    f = lambda v: np.array(v, dtype=np.float32)
    for variant, nbits in ((RNE, 0), (SRFF, 2), (SRC, 3), (TA, 0)):
        got = oracle.round_format16(f([65504.0, 65519.0, 65520.0, 70000.0, -65519.0, -65520.0, np.inf, -np.inf]), FROM_FP32,
                                    BINARY16, variant, nbits, seed=1)
        assert list(got) == [0x7BFF, 0x7BFF, 0x7C00, 0x7C00, 0xFBFF, 0xFC00, 0x7C00, 0xFC00], variant
        d = E5M6_SAT
        M = float(value_of(d[3], d))
        got = oracle.round_format16(f([M, M * 1.5, -M * 4, np.inf, -np.inf, np.nan]), FROM_FP32, d, variant, nbits, seed=1)
        assert list(got[:5]) == [d[3], d[3], d[3] | 0x800, d[3], d[3] | 0x800] and (got[5] & 0x7FF) == d[3], variant
    assert list(oracle.round_format16(f([np.nan]), FROM_FP32, E6M9, RNE, 0, seed=0)) == [E6M9[5]]


@pytest.mark.parametrize("src", [FROM_BF16, FROM_FP16, FROM_FP32])
def test_array_call_is_the_per_element_rule(oracle, src):
    rng = np.random.default_rng(8)
    n = 3000
    if src == FROM_FP32:
        x = (rng.standard_normal(n) * 2.0 ** rng.integers(-20, 14, n)).astype(np.float32)
        vals = x
    else:
        x = rng.integers(0, 1 << 16, n, dtype=np.uint16)
        vals = np.array([oracle.widen16(int(c), src) for c in x], dtype=np.uint32).view(np.float32)
    for d in (BINARY16, E6M9):
        for variant, nbits in ((SRFF, 3), (SRF, 7), (SRC, 2), (SRC_ODD, 4), (RNE, 0)):
            got = oracle.round_format16(x, src, d, variant, nbits, seed=12, offset=1000)
            for j in list(range(0, n, 97)) + [n - 1]:
                if np.isnan(vals[j]):
                    continue
                r = oracle.random_bits(12, 0, 1000 + j, nbits) if variant in DRAWING else 0
                assert got[j] == oracle.round_format16_with_n(vals[j], d, variant, nbits, r)
