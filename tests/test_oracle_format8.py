"""Pins for the oracle's generic-format path (any (K, P, B; M) of Sec. II with K <= 8, the extra
rounding modes of Sec. II-A / Sec. III-F): published value sets, the already pinned fixed-format
path, library roundings, exact counting arguments and the closed-form biases of Sec. III.
Nothing here touches the GPU library.  CPU only."""
import bisect
import math
from fractions import Fraction

import numpy as np
import pytest

from exact_model import expected_ups, f32_fraction, floor_frac, pow2

RNE, SRFF, SRF, SRC, SRC_ODD, TNO, TA = range(7)
DRAWING = (SRFF, SRF, SRC, SRC_ODD)
FROM_BF16, FROM_FP16, FROM_FP32 = 0, 1, 2


# Descriptors (K, P, B, max_code, inf_code, nan_code, nan_signed, neg_zero), written here from the
# formats' public definitions -- OCP 8-bit floating point (E4M3: S.1111.111 is NaN, no infinity;
# E5M2: IEEE-like), OCP microscaling element types (E3M2, E2M3, E2M1: no NaN, no infinity), and the
# IEEE WG P3109 interim report's binary8pP (bias 2^(7-P), 0x80 the only NaN, 0x7F / 0xFF the
# infinities, no negative zero) whose binary8p4 is the format Sec. IV trains in.
def p3109(P):
    return (8, P, 1 << (7 - P), 0x7E, 0x7F, 0x80, 0, 0)


E4M3 = (8, 4, 7, 0x7E, -1, 0x7F, 1, 1)
E5M2 = (8, 3, 15, 0x7B, 0x7C, 0x7E, 1, 1)
E3M2 = (6, 3, 3, 0x1F, -1, -1, 0, 1)
E2M3 = (6, 4, 1, 0x1F, -1, -1, 0, 1)
E2M1 = (4, 2, 1, 0x07, -1, -1, 0, 1)
BINARY8P4 = p3109(4)
ALL = {"e4m3": E4M3, "e5m2": E5M2, "e3m2": E3M2, "e2m3": E2M3, "e2m1": E2M1, "binary8p1": p3109(1),
       "binary8p3": p3109(3), "binary8p4": BINARY8P4, "binary8p5": p3109(5), "binary8p7": p3109(7)}


def value_of(code, d):
    """Eq. (1) for a non-negative finite magnitude code, as a Fraction."""
    K, P, B = d[0], d[1], d[2]
    e, t = code >> (P - 1), code & ((1 << (P - 1)) - 1)
    if e == 0:
        return Fraction(t) * pow2(1 - P) * pow2(1 - B)
    return (1 + Fraction(t) * pow2(1 - P)) * pow2(e - B)


_TABLES = {}


def table(d):
    key = tuple(int(v) for v in d)
    if key not in _TABLES:
        vals = [value_of(c, d) for c in range(d[3] + 1)]
        assert vals == sorted(vals)
        _TABLES[key] = vals
    return _TABLES[key]


def position(a, d):
    """(lower magnitude code, delta in [0,1)) of the Fraction 0 <= a <= M."""
    vals = table(d)
    i = bisect.bisect_right(vals, a) - 1
    if vals[i] == a:
        return i, Fraction(0)
    return i, (a - vals[i]) / (vals[i + 1] - vals[i])


def rno_int(q):
    f = floor_frac(q)
    r = q - f
    if r > Fraction(1, 2) or (r == Fraction(1, 2) and f % 2 == 0):
        return f + 1
    return f


def ups(delta, variant, N):
    if variant == SRC_ODD:
        return min(rno_int(delta * 2 ** N), 2 ** N)
    return expected_ups(delta, variant, N)


def inputs_below_max(rng, d, count):
    """fp32 values over the whole finite range of the format, sub-subnormal magnitudes included."""
    K, P, B, max_code = d[:4]
    lo = 127 + (1 - B) - (P - 1) - 3
    hi = 127 + ((max_code >> (P - 1)) - B)
    bits = rng.integers(0, 1 << 32, size=count, dtype=np.uint32)
    field = rng.integers(max(lo, 1), hi + 1, size=count, dtype=np.uint32)
    x = ((bits & np.uint32(0x807FFFFF)) | (field << np.uint32(23))).view(np.float32)
    M = float(value_of(max_code, d))
    return x[np.abs(x.astype(np.float64)) <= M]


# ------------------------------------------------------------------ published value sets ----
def test_published_value_sets(oracle):
    dec = oracle.decode_format8
    assert [dec(c, E2M1) for c in range(8)] == [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    assert [dec(c | 8, E2M1) for c in range(1, 8)] == [-0.5, -1.0, -1.5, -2.0, -3.0, -4.0, -6.0]
    assert dec(0x1F, E2M3) == 7.5 and dec(0x01, E2M3) == 0.125 and dec(0x08, E2M3) == 1.0
    assert dec(0x1F, E3M2) == 28.0 and dec(0x01, E3M2) == 0.0625 and dec(0x0C, E3M2) == 1.0
    assert dec(0x7E, E4M3) == 448.0 and dec(0x01, E4M3) == 2.0 ** -9 and math.isnan(dec(0x7F, E4M3)) and math.isnan(dec(0xFF, E4M3))
    assert dec(0x7B, E5M2) == 57344.0 and dec(0x01, E5M2) == 2.0 ** -16 and dec(0x7C, E5M2) == math.inf and dec(0xFC, E5M2) == -math.inf
    assert all(math.isnan(dec(c, E5M2)) for c in (0x7D, 0x7E, 0x7F, 0xFD))
    # binary8p4: 1.0 is 0x40, the largest finite value 224, the smallest subnormal 2^-10
    assert dec(0x40, BINARY8P4) == 1.0 and dec(0x7E, BINARY8P4) == 224.0 and dec(0x01, BINARY8P4) == 2.0 ** -10
    assert dec(0x08, BINARY8P4) == 2.0 ** -7 and dec(0xC0, BINARY8P4) == -1.0
    assert dec(0x7F, BINARY8P4) == math.inf and dec(0xFF, BINARY8P4) == -math.inf and math.isnan(dec(0x80, BINARY8P4))
    assert dec(0x00, BINARY8P4) == 0.0 and not math.copysign(1.0, dec(0x00, BINARY8P4)) < 0
    assert dec(0x7E, p3109(3)) == 49152.0 and dec(0x7E, p3109(5)) == 15.0
    assert dec(0x7E, p3109(1)) == 2.0 ** 62 and dec(0x01, p3109(1)) == 2.0 ** -63 and dec(0x40, p3109(1)) == 1.0
    assert dec(0x7E, p3109(7)) == 1.0 + 62.0 / 64.0 and dec(0x01, p3109(7)) == 1.0 / 64.0


@pytest.mark.parametrize("name", sorted(ALL))
def test_decode_is_eq1_on_every_code(oracle, name):
    d = ALL[name]
    K = d[0]
    for code in range(1 << K):
        mag, neg = code & ((1 << (K - 1)) - 1), code >> (K - 1)
        got = oracle.decode_format8(code, d)
        special = (mag > d[3]) or (code == d[5]) or (d[6] and mag == d[5]) or (mag == 0 and neg and not d[7])
        if special:
            assert math.isnan(got) or (mag == d[4] and math.isinf(got) and (got < 0) == bool(neg)), (name, code)
        else:
            assert Fraction(got) == (-1 if neg else 1) * value_of(mag, d), (name, code)


def test_descriptor_validation(oracle):
    assert all(oracle.format8_check(d) for d in ALL.values())
    bad = [(9, 4, 7, 0x7E, -1, 0x7F, 1, 1), (8, 8, 7, 0x7E, -1, 0x7F, 1, 1), (8, 0, 7, 0x7E, -1, 0x7F, 1, 1),
           (8, 4, 7, 0x80, -1, -1, 0, 1),          # max_code outside the magnitude range
           (8, 4, 7, 0x03, -1, -1, 0, 1),          # M would be subnormal
           (8, 4, 7, 0x7E, 0x7E, -1, 0, 1),        # infinity not above M
           (8, 4, 7, 0x7E, -1, 0x7E, 0, 1),        # NaN on a finite code
           (8, 4, 7, 0x7E, -1, 0x80, 0, 1),        # 0x80 is -0 in a format with negative zero
           (8, 4, 7, 0x7E, 0x7F, 0x7F, 0, 1),      # NaN on the infinity
           (8, 4, 97, 0x7E, -1, 0x7F, 1, 1),       # bias out of range
           (8, 1, 0, 0x7F, -1, -1, 0, 1)]          # M + ulp(M) beyond fp32
    assert not any(oracle.format8_check(d) for d in bad)


def random_descriptors(rng, count, check):
    """Valid descriptors drawn at random (rejection against `check`), special encodings of every kind included."""
    out = []
    while len(out) < count:
        K = int(rng.integers(2, 9))
        P = int(rng.integers(1, K))
        top = (1 << (K - 1)) - 1
        mx = int(rng.integers(1 << (P - 1), top + 1))
        B = int(rng.integers(0, 41))
        inf = int(rng.integers(mx + 1, top + 1)) if mx < top and rng.random() < 0.5 else -1
        neg_zero = int(rng.random() < 0.6)
        kind = rng.random()
        if kind < 0.3:
            nan, signed = -1, 0
        elif kind < 0.45 and not neg_zero:
            nan, signed = 1 << (K - 1), 0
        else:
            spare = [m for m in range(mx + 1, top + 1) if m != inf]
            if not spare:
                continue
            nan, signed = int(rng.choice(spare)), int(rng.random() < 0.5)
            if not signed and rng.random() < 0.3:
                nan |= 1 << (K - 1)
        d = (K, P, B, mx, inf, nan, signed, neg_zero)
        if check(d):
            out.append(d)
    return out


def test_random_descriptors_bracket_count_and_fix(oracle):
    """Forty descriptors drawn at random: every rounded magnitude is a bracketing neighbour from the exact table of
    Eq. (1), the number of draws that round up is the counting argument, representable values stay, and out-of-range
    and special inputs follow the descriptor."""
    rng = np.random.default_rng(2024)
    for d in random_descriptors(rng, 40, oracle.format8_check):
        K, P, B, mx, inf, nan, signed, neg_zero = d
        sign_bit = 1 << (K - 1)
        vals = table(d)
        for xv in inputs_below_max(rng, d, 40):
            a = abs(f32_fraction(xv))
            lo, delta = position(a, d)
            for variant in DRAWING:
                N = int(rng.integers(1, 6))
                got = sum((oracle.round_format8_with_n(xv, d, variant, N, n) & (sign_bit - 1)) == lo + 1 for n in range(1 << N))
                assert got == (ups(delta, variant, N) if delta != 0 else 0), (d, xv, variant, N)
            for variant in (RNE, TNO, TA):
                code = oracle.round_format8_with_n(xv, d, variant, 0, 0)
                assert (code & (sign_bit - 1)) in ((lo,) if delta == 0 else (lo, lo + 1)), (d, xv, variant)
                if (code & (sign_bit - 1)) == 0 and not neg_zero:
                    assert code == 0
        for code in range(0, mx + 1, max(1, mx // 16)):
            assert oracle.round_format8_with_n(np.float32(float(vals[code])), d, SRFF, 3, 7) == code
        M = float(vals[mx])
        big = oracle.round_format8_with_n(np.float32(M * 4.0), d, SRC, 3, 5)
        assert big == (inf if inf >= 0 else mx), d
        neg_nan = np.array([0xFFC00000], dtype=np.uint32).view(np.float32)[0]
        got = oracle.round_format8_with_n(neg_nan, d, SRF, 3, 1)
        assert got == ((nan | (sign_bit if signed else 0)) if nan >= 0 else (mx | sign_bit)), d


# ------------------------------------------------------ against the pinned fixed-format path ----
@pytest.mark.parametrize("fmt,d", [(1, E4M3), (2, E5M2)])
def test_descriptor_path_equals_fixed_path(oracle, fmt, d):
    rng = np.random.default_rng(11 + fmt)
    x = rng.integers(0, 1 << 32, size=4000, dtype=np.uint32).view(np.float32)
    M = oracle.decode_format8(d[3], d)
    ulp_M = M - oracle.decode_format8(d[3] - 1, d)
    edge = np.array([0.0, -0.0, M, -M, M + ulp_M / 2, -(M + ulp_M / 2), np.nextafter(np.float32(M + ulp_M / 2), np.float32(0)),
                     np.nextafter(np.float32(M + ulp_M / 2), np.float32(np.inf)), np.inf, -np.inf, np.nan, -np.nan,
                     2.0 ** -149, -2.0 ** -149, 2.0 ** -126], dtype=np.float32)
    edge[11] = np.array([0xFFC00001], dtype=np.uint32).view(np.float32)[0]   # a negative NaN with a payload
    x = np.concatenate([x, edge, inputs_below_max(rng, d, 4000)])
    for variant in (RNE, SRFF, SRF, SRC):
        for nbits in (1, 3, 8, 16):
            ns = rng.integers(0, 1 << nbits, size=x.size)
            for xv, n in zip(x, ns):
                assert oracle.round_format8_with_n(xv, d, variant, nbits, int(n)) == oracle.round_with_n(xv, fmt, variant, nbits, int(n)), (xv, variant, nbits, n)
            if variant == RNE:
                break
    for code in range(256):
        a, b = oracle.decode_format8(code, d), oracle.decode(code, fmt)
        assert (math.isnan(a) and math.isnan(b)) or a == b


# ----------------------------------------------------------- bracketing, identity, counting ----
@pytest.mark.parametrize("name", sorted(ALL))
def test_bracket_and_identity(oracle, name):
    d = ALL[name]
    rng = np.random.default_rng(5)
    vals = table(d)
    for xv in inputs_below_max(rng, d, 300):
        a = abs(f32_fraction(xv))
        lo, delta = position(a, d)
        for variant in range(7):
            nbits = int(rng.integers(1, 9))
            n = int(rng.integers(0, 1 << nbits))
            code = oracle.round_format8_with_n(xv, d, variant, nbits, n)
            mag, neg = code & ((1 << (d[0] - 1)) - 1), code >> (d[0] - 1)
            assert mag in ((lo,) if delta == 0 else (lo, lo + 1)), (name, xv, variant)
            if mag != 0 or d[7]:
                assert neg == int(np.signbit(xv))
            else:
                assert neg == 0          # no negative zero in this format
    for code in range(d[3] + 1):         # representable values never move, whatever is drawn
        xv = np.float32(float(vals[code]))
        for variant in range(7):
            for n in (0, 1, 7):
                assert oracle.round_format8_with_n(xv, d, variant, 3, n) == code
                neg = oracle.round_format8_with_n(-xv, d, variant, 3, n)
                assert neg == (code | (1 << (d[0] - 1)) if (code or d[7]) else 0)


@pytest.mark.parametrize("name", ["binary8p4", "binary8p3", "e2m3", "e2m1", "binary8p1", "binary8p7"])
@pytest.mark.parametrize("variant", DRAWING)
def test_exhaustive_round_up_counts(oracle, name, variant):
    """For every draw n of N bits: the number that round away from zero equals the counting argument
    over the exact delta (target subnormals and values below the smallest subnormal included)."""
    d = ALL[name]
    rng = np.random.default_rng(17)
    for xv in inputs_below_max(rng, d, 60):
        a = abs(f32_fraction(xv))
        lo, delta = position(a, d)
        for N in (1, 2, 3, 5):
            got = sum((oracle.round_format8_with_n(xv, d, variant, N, n) & ((1 << (d[0] - 1)) - 1)) == lo + 1
                      for n in range(1 << N))
            want = ups(delta, variant, N) if delta != 0 else 0
            assert got == want, (name, xv, variant, N, got, want)


@pytest.mark.parametrize("name", ["binary8p4", "e5m2", "e2m1", "binary8p1", "binary8p7"])
@pytest.mark.parametrize("N", [17, 20, 23, 24])
def test_round_up_threshold_with_many_bits(oracle, name, N):
    """With 17 to 24 bits the draws are too many to count one by one, but every variant rounds up for exactly the
    largest draws: with U = the counting argument's number over the exact delta, n = 2^N - U is the first draw that
    rounds up and the one before it the last that does not.  Inputs reach below the smallest subnormal, where delta
    carries more bits than any fixed-point word of the kernels holds, and half of them have short significands (ties
    of the inner rounding of Eq. (7))."""
    d = ALL[name]
    rng = np.random.default_rng(100 + N)
    x = inputs_below_max(rng, d, 50)
    short = inputs_below_max(rng, d, 50).view(np.uint32) & np.uint32(0xFFFF0000)
    mask = (1 << (d[0] - 1)) - 1
    for xv in np.concatenate([x, short.view(np.float32)]):
        a = abs(f32_fraction(xv))
        lo, delta = position(a, d)
        for variant in DRAWING:
            U = ups(delta, variant, N) if delta != 0 else 0
            first_up = (1 << N) - U
            probes = {0: lo if U < (1 << N) else lo + 1, (1 << N) - 1: lo + 1 if U > 0 else lo}
            if U > 0:
                probes[first_up] = lo + 1
                probes[int(rng.integers(first_up, 1 << N))] = lo + 1
            if first_up > 0:
                probes[first_up - 1] = lo
                probes[int(rng.integers(0, first_up))] = lo
            for n, want in probes.items():
                got = oracle.round_format8_with_n(xv, d, variant, N, n) & mask
                assert got == want, (name, float(xv), variant, N, n, got, want, U)


@pytest.mark.parametrize("N", [1, 2, 3, 4])
def test_src_with_ties_to_odd_is_unbiased_and_differs_only_at_ties(oracle, N):
    """Sec. III-F allows ties-to-even or ties-to-odd for SRC's inner rounding: over a full grid of
    D = 6 excess bits the mean of (P(up) - delta) is exactly zero for both, and the two variants
    disagree only where delta 2^N lies exactly half-way."""
    d = BINARY8P4                      # ulp 2^-3 in [1, 2): x = 1 + k 2^-9 gives D = 6
    total = {SRC: Fraction(0), SRC_ODD: Fraction(0)}
    for k in range(64):
        xv = np.float32(1.0 + k * 2.0 ** -9)
        delta = Fraction(k, 64)
        cnt = {}
        for variant in (SRC, SRC_ODD):
            cnt[variant] = sum(oracle.round_format8_with_n(xv, d, variant, N, n) == 0x41 for n in range(1 << N))
            total[variant] += Fraction(cnt[variant], 1 << N) - delta
        tie = (delta * 2 ** N) % 1 == Fraction(1, 2)
        assert (cnt[SRC] != cnt[SRC_ODD]) == tie, (k, cnt)
    assert total[SRC] == 0 and total[SRC_ODD] == 0


# ------------------------------------------------------------- deterministic modes vs library ----
def test_deterministic_modes_on_an_integer_grid(oracle):
    """In [8, 16) E4M3's ulp is 1, so rounding to the format is rounding to an integer: ties-to-even is
    numpy's rint, ties-away (Eq. (4)) is floor(x + 1/2), ties-to-odd picks the odd neighbour of a tie."""
    d = E4M3
    for k in range(64, 128):
        xv = np.float32(k / 8.0)
        want_even = int(np.rint(np.float64(xv)))
        want_away = int(np.floor(np.float64(xv) + 0.5))
        is_tie = (k % 8) == 4
        want_odd = want_even if not is_tie else (want_even + 1 if want_even == int(np.floor(xv)) else want_even - 1)
        if is_tie:
            assert want_odd % 2 == 1 and want_even % 2 == 0
        for sign in (1.0, -1.0):     # sign-magnitude: "away" is away from zero
            got = {v: sign * oracle.decode_format8(oracle.round_format8_with_n(sign * xv, d, v, 0, 0), d) for v in (RNE, TNO, TA)}
            assert got[RNE] == want_even and got[TA] == want_away and got[TNO] == want_odd, (k, got)


# ----------------------------------------------------------------- overflow and specials ----
def test_overflow_and_specials(oracle):
    r = lambda x, d, v=SRFF, N=3, n=0: oracle.round_format8_with_n(np.float32(x), d, v, N, n)
    up = lambda v: np.nextafter(np.float32(v), np.float32(np.inf))
    down = lambda v: np.nextafter(np.float32(v), np.float32(0))
    for v in range(7):
        for n in (0, 7):
            # binary8p4: M = 224 = 14 * 16 has an even significand, so the tie 232 stays finite
            assert r(232.0, BINARY8P4, v, 3, n) == 0x7E and r(-232.0, BINARY8P4, v, 3, n) == 0xFE
            assert r(up(232.0), BINARY8P4, v, 3, n) == 0x7F and r(down(232.0), BINARY8P4, v, 3, n) == 0x7E
            assert r(up(224.0), BINARY8P4, v, 3, n) == 0x7E          # above M: no draw can reach infinity
            assert r(np.inf, BINARY8P4, v, 3, n) == 0x7F and r(-np.inf, BINARY8P4, v, 3, n) == 0xFF
            assert r(np.nan, BINARY8P4, v, 3, n) == 0x80 and r(-np.nan, BINARY8P4, v, 3, n) == 0x80
            assert r(0.0, BINARY8P4, v, 3, n) == 0x00 and r(-0.0, BINARY8P4, v, 3, n) == 0x00
            # E5M2: M = 57344 = 7 * 8192 has an odd significand, the tie 61440 goes to infinity
            assert r(61440.0, E5M2, v, 3, n) == 0x7C and r(down(61440.0), E5M2, v, 3, n) == 0x7B
            # binary8p3: M = 49152 = 6 * 8192: even
            assert r(49152.0 + 4096.0, p3109(3), v, 3, n) == 0x7E and r(up(49152.0 + 4096.0), p3109(3), v, 3, n) == 0x7F
            # saturating formats
            assert r(100.0, E2M1, v, 3, n) == 0x7 and r(-np.inf, E2M1, v, 3, n) == 0xF and r(np.inf, E4M3, v, 3, n) == 0x7E
            assert r(1e30, E3M2, v, 3, n) == 0x1F and r(-7.75, E2M3, v, 3, n) == 0x3F
            assert r(np.nan, E4M3, v, 3, n) == 0x7F and r(-np.nan, E4M3, v, 3, n) == 0xFF
            assert r(np.nan, E2M1, v, 3, n) == 0x7 and r(-np.nan, E2M1, v, 3, n) == 0xF      # no NaN code: +-M
            assert r(-0.0, E4M3, v, 3, n) == 0x80
    # a small negative value that rounds to zero: -0 where the format has it, 0 where it has not
    assert r(-2.0 ** -20, BINARY8P4, SRFF, 3, 0) == 0x00 and r(-2.0 ** -20, E4M3, SRFF, 3, 0) == 0x80
    assert r(-2.0 ** -11, BINARY8P4, RNE) == 0x00 and r(-2.0 ** -11, BINARY8P4, TA) == 0x81 and r(-2.0 ** -11, BINARY8P4, TNO) == 0x81


# ------------------------------------------------------- the narrow-source training setting ----
@pytest.mark.parametrize("N", [1, 2, 3, 4, 5])
def test_bf16_to_binary8p4_closed_form_biases(oracle, N):
    """Sec. IV's setting: bf16 updates (precision 8) into binary8p4 (precision 4), D = 4 excess bits,
    3 random bits used, 4 ideal.  Over all bf16 values of one binade and all draws, the mean error in
    target ulps is (2^-D - 2^-N)/2 for SRFF, 2^-(D+1) for SRF (both 0 once N >= D) and 0 for SRC."""
    d = BINARY8P4
    D = 4
    codes16 = np.arange(0x3F80, 0x4000, dtype=np.uint16)        # bf16 values in [1, 2)
    x = (codes16.astype(np.uint32) << 16).view(np.float32)
    want = {SRFF: (Fraction(1, 2 ** D) - Fraction(1, 2 ** N)) / 2 if N < D else Fraction(0),
            SRF: Fraction(1, 2 ** (D + 1)) if N < D else Fraction(0), SRC: Fraction(0), SRC_ODD: Fraction(0)}
    for variant in DRAWING:
        err = Fraction(0)
        for xv in x:
            for n in range(1 << N):
                y = oracle.decode_format8(oracle.round_format8_with_n(xv, d, variant, N, n), d)
                err += (Fraction(y) - Fraction(float(xv))) / Fraction(1, 8)
        assert err / (x.size << N) == want[variant], (variant, N)


# ------------------------------------------------------------ per-bin statistics (Figs. 1-2) ----
@pytest.mark.parametrize("fmt,d", [(1, E4M3), (2, E5M2)])
def test_stats_under_an_ocp_descriptor_equal_the_fixed_format_statistics(oracle, fmt, d):
    """The descriptor form of the per-bin statistics against the fixed-format one (pinned on its own): same codes,
    same four sums bit for bit, on inputs from below the smallest subnormal to beyond M with NaN and infinities."""
    rng = np.random.default_rng(61 + fmt)
    x = np.concatenate([inputs_below_max(rng, d, 6000), rng.integers(0, 1 << 32, size=1500, dtype=np.uint32).view(np.float32),
                        np.array([np.inf, -np.inf, np.nan, 0.0, -0.0], dtype=np.float32)])
    for variant, nbits in ((RNE, 0), (SRFF, 2), (SRF, 3), (SRC, 3), (SRC, 11), (SRFF, 20)):
        for group, offset in ((500, 0), (1 << 20, 12345), (7, 3), (500, 5000)):
            first = offset // group
            nbins = (offset + x.size - 1) // group - first + 1
            a, ca = oracle.bias_stats_format8(x, d, variant, nbits, 9, offset, group, first, nbins, want_out=True)
            b, cb = oracle.bias_stats(x, fmt, variant, nbits, 9, offset, group, first, nbins, want_out=True)
            assert np.array_equal(ca, cb)
            assert np.array_equal(a, b, equal_nan=True), (variant, nbits, group)


@pytest.mark.parametrize("name", ["binary8p3", "binary8p4", "e2m3", "e2m1", "binary8p1", "binary8p7"])
def test_stats_sums_are_the_exact_rational_sums(oracle, name):
    """{count, sum y, sum e, sum e^2} per bin against sums of exact rationals: y from Eq. (1) on the returned code
    (value_of above), ulp_t(x) = 2^(max(floor(log2 |x|), 1 - B) - P + 1) from Eq. (2) by integer arithmetic on x's
    own fraction, e = (y - x) / ulp_t(x); normal and subnormal range, far below the smallest subnormal, both signs,
    zeros, and the range above M of the formats that saturate (y = +-M)."""
    d = ALL[name]
    K, P, B, max_code, inf_code = d[:5]
    M = value_of(max_code, d)
    rng = np.random.default_rng(abs(hash(name)) % 1000)
    group = 300
    fM = float(M)
    parts = [rng.uniform(2.0 ** (1 - B), fM, group), rng.uniform(2.0 ** (-B - P - 20), 2.0 ** (1 - B), group),
             -np.exp(rng.uniform(np.log(2.0 ** (-B - P - 3)), np.log(fM), group)),
             np.concatenate([np.zeros(5), -np.zeros(5), rng.uniform(2.0 ** -B, min(2.0 ** (3 - B), fM), group - 10)])]
    if inf_code < 0:
        parts.append(rng.uniform(fM, 8 * fM, group) * np.where(rng.integers(0, 2, group) == 1, -1.0, 1.0))
    x = np.concatenate(parts).astype(np.float32)
    nbins = len(parts)
    for variant, nbits in ((SRFF, 2), (SRF, 3), (SRC, 3), (RNE, 0), (SRC_ODD, 4), (TA, 0)):
        stats, out = oracle.bias_stats_format8(x, d, variant, nbits, 6, 0, group, 0, nbins, want_out=True)
        for b in range(nbins):
            sy = se = see = Fraction(0)
            for j in range(b * group, (b + 1) * group):
                xf = f32_fraction(x[j])
                code = int(out[j])
                mag = code & ((1 << (K - 1)) - 1)
                assert mag <= max_code
                y = value_of(mag, d) * (-1 if code >> (K - 1) else 1)
                a = abs(xf)
                lg = (a.numerator.bit_length() - a.denominator.bit_length()) if a else 1 - B
                if a and Fraction(2) ** lg > a:
                    lg -= 1
                e = (y - xf) / Fraction(2) ** (max(lg, 1 - B) - P + 1)
                sy, se, see = sy + y, se + e, see + e * e
            assert stats[b, 0] == group
            assert abs(stats[b, 1] - float(sy)) <= 1e-13 * abs(float(sy)), (name, variant, b)
            assert abs(stats[b, 2] - float(se)) <= 1e-12 * max(abs(float(se)), 1.0), (name, variant, nbits, b)
            assert abs(stats[b, 3] - float(see)) <= 1e-12 * float(see), (name, variant, nbits, b)


def test_stats_of_bf16_values_into_binary8p4_give_the_closed_form_biases(oracle):
    """Sec. III-E through the statistics entry: all bf16 values of [1, 2) (D = 4 excess bits for binary8p4) repeated
    over many draws; the per-bin mean of e tends to (2^-D - 2^-N)/2 for SRFF, 2^-(D+1) for SRF and 0 for SRC."""
    d, D, N = BINARY8P4, 4, 3
    x = np.tile((np.arange(0x3F80, 0x4000, dtype=np.uint32) << 16).view(np.float32), 4096)
    want = {SRFF: (2.0 ** -D - 2.0 ** -N) / 2, SRF: 2.0 ** -(D + 1), SRC: 0.0, SRC_ODD: 0.0}
    for variant in DRAWING:
        stats, _ = oracle.bias_stats_format8(x, d, variant, N, 3, 0, x.size, 0, 1)
        assert stats[0, 0] == x.size
        assert abs(stats[0, 2] / x.size - want[variant]) < 2e-3, (variant, stats[0, 2] / x.size)   # five standard errors
        assert abs(stats[0, 1] / x.size - (1.5 - 2.0 ** -8 + want[variant] / 8)) < 2.5e-4


def test_stats_reject_bad_arguments_and_elements_outside_the_bins(oracle):
    x = np.ones(10, dtype=np.float32)
    for bad in (lambda: oracle.bias_stats_format8(x, (9, 4, 7, 0x7E, -1, 0x7F, 1, 1), SRFF, 2, 1, 0, 5, 0, 2),
                lambda: oracle.bias_stats_format8(x, BINARY8P4, SRFF, 0, 1, 0, 5, 0, 2),
                lambda: oracle.bias_stats_format8(x, BINARY8P4, SRFF, 2, 1, 0, 0, 0, 2),
                lambda: oracle.bias_stats_format8(x, BINARY8P4, SRFF, 2, 1, 0, 5, 0, 1),
                lambda: oracle.bias_stats_format8(x, BINARY8P4, SRFF, 2, 1, 0, 5, 1, 2)):
        with pytest.raises(ValueError):
            bad()


# --------------------------------------------------------------------------- array entry ----
@pytest.mark.parametrize("src", [FROM_BF16, FROM_FP16, FROM_FP32])
def test_array_call_is_the_per_element_rule(oracle, src):
    rng = np.random.default_rng(23 + src)
    n = 3000
    if src == FROM_FP32:
        x = rng.integers(0, 1 << 32, size=n, dtype=np.uint32).view(np.float32)
        wide = x
    else:
        x = rng.integers(0, 1 << 16, size=n, dtype=np.uint16)
        wide = np.array([oracle.widen16(int(c), src) for c in x], dtype=np.uint32).view(np.float32)
    for name in ("binary8p4", "e2m3"):
        d = ALL[name]
        for variant, nbits in ((RNE, 0), (SRFF, 3), (SRF, 2), (SRC, 5), (SRC_ODD, 3), (TNO, 0), (TA, 0)):
            seed, offset = 77, 12345
            got = oracle.round_format8(x, src, d, variant, nbits, seed, offset)
            for j in range(0, n, 7):
                r = oracle.random_bits(seed, 0, offset + j, nbits) if variant in DRAWING else 0
                assert got[j] == oracle.round_format8_with_n(wide[j], d, variant, nbits, r), (name, variant, j)
            # chunked == whole (the bits are a function of the global index)
            part = oracle.round_format8(x[1000:], src, d, variant, nbits, seed, offset + 1000)
            assert np.array_equal(part, got[1000:])


# ------------------------------------------------------------------ fused QAT step, generic ----
def _bf16_codes(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def _bf16_values(c):
    return (np.asarray(c, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


@pytest.mark.parametrize("fmt,d", [(1, E4M3), (2, E5M2)])
def test_qat_step_with_ocp_descriptor_equals_the_fixed_path(oracle, fmt, d):
    """The generic-format step only swaps the 8-bit decode and the 8-bit rounding; with the descriptor of
    an OCP fp8 format it must reproduce the fixed-format step (pinned against a library AdamW) on every
    input, NaN codes and wild moments included."""
    rng = np.random.default_rng(3 + fmt)
    n = 6000
    w8 = rng.integers(0, 256, n).astype(np.uint8)
    g16 = _bf16_codes(rng.standard_normal(n) * 0.3)
    m16 = _bf16_codes(rng.standard_normal(n) * 0.05)
    v16 = _bf16_codes(rng.random(n) * 0.02)
    k = n // 4
    g16[:k] = rng.integers(0, 1 << 16, k)
    m16[k:2 * k] = rng.integers(0, 1 << 16, k)
    v16[2 * k:3 * k] = rng.integers(0, 1 << 16, k)
    for params in ((1e-3, 0.9, 0.999, 1e-8, 0.01, 0.1, 0.001), (0.5, 0.0, 0.5, 1e-3, 0.0, 1.0, 0.5)):
        for variant, nbits in ((RNE, 0), (SRFF, 3), (SRF, 3), (SRC, 4)):
            a = oracle.qat_adamw_step(w8, g16, m16, v16, fmt, params, variant, nbits, seed=7, step=5, offset=9)
            b = oracle.qat_adamw_step_format8(w8, g16, m16, v16, d, params, variant, nbits, seed=7, step=5, offset=9)
            for x, y in zip(a, b):
                assert np.array_equal(x, y)


def test_qat_step_structure_in_binary8p4(oracle):
    """Sec. IV's configuration (binary8p4 weights, bf16 updates).  lr = 0 leaves every finite weight where
    it is; the stored weight is the generic narrow-source rounding of the bf16 sum, recomputed here in
    numpy fp32, with the bits of (seed, step, index); a NaN sum is stored as 0x80; the format's missing
    negative zero shows when a small negative weight is pulled to zero."""
    d = BINARY8P4
    rng = np.random.default_rng(4)
    n = 3000
    w8 = rng.integers(0, 256, n).astype(np.uint8)
    w8[w8 == 0x80] = 0x00                      # NaN
    w8[(w8 & 0x7F) == 0x7F] ^= 0x01            # infinities -> the largest finite value
    g16 = _bf16_codes(rng.standard_normal(n))
    m16 = _bf16_codes(rng.standard_normal(n) * 0.1)
    v16 = _bf16_codes(rng.random(n) * 0.1)
    for variant, nbits in ((RNE, 0), (SRFF, 3), (SRF, 3), (SRC, 3), (SRC_ODD, 3), (TNO, 0), (TA, 0)):
        same, _, _ = oracle.qat_adamw_step_format8(w8, g16, m16, v16, d, (0.0, 0.9, 0.999, 1e-8, 0.01, 0.1, 0.001), variant, nbits, 1, 4)
        assert np.array_equal(same, w8)
    w = np.array([oracle.decode_format8(int(c), d) for c in w8], dtype=np.float32)
    for variant, nbits in ((SRF, 3), (SRC_ODD, 3), (TA, 0)):
        seed, step, off = 11, 6, 40
        lr, b1, b2, eps, wd, c1, c2 = (np.float32(v) for v in (0.05, 0.9, 0.99, 1e-8, 0.1, 0.3, 0.05))
        g, m0, v0 = _bf16_values(g16), _bf16_values(m16), _bf16_values(v16)
        one = np.float32(1.0)
        fma = lambda a, b, c: (a.astype(np.float64) * b.astype(np.float64) + c.astype(np.float64)).astype(np.float32)
        m1 = fma(np.full(n, b1), m0, (one - b1) * g)
        v1 = fma(np.full(n, b2), v0, (one - b2) * (g * g))
        mq, vq = _bf16_values(_bf16_codes(m1)), _bf16_values(_bf16_codes(v1))
        ratio = (mq / c1) / (np.sqrt(vq / c2) + eps)
        u = -lr * fma(np.full(n, wd), w, ratio)
        s16 = _bf16_values(_bf16_codes(w + _bf16_values(_bf16_codes(u))))
        got, _, _ = oracle.qat_adamw_step_format8(w8, g16, m16, v16, d, (lr, b1, b2, eps, wd, c1, c2), variant, nbits, seed, step, off)
        want = np.array([oracle.round_format8_with_n(x, d, variant, nbits, oracle.random_bits(seed, step, off + j, nbits) if variant in DRAWING else 0)
                         for j, x in enumerate(s16)], dtype=np.uint8)
        assert np.array_equal(got, want)
    # specials: a NaN weight or gradient gives the NaN code; a huge update reaches the infinity code
    w_nan = np.array([0x80, 0x40, 0x40, 0x89], dtype=np.uint8)
    g_sp = np.array([0x3F80, 0x7FC0, 0x3F80, 0xBF80], dtype=np.uint16)       # 1.0, NaN, 1.0, -1.0
    z = np.zeros(4, np.uint16)
    out, _, _ = oracle.qat_adamw_step_format8(w_nan, g_sp, z, z, d, (1e30, 0.9, 0.999, 1e-8, 0.0, 0.1, 0.001), RNE, 0, 0, 1)
    assert list(out) == [0x80, 0x80, 0xFF, 0x7F]
    # the smallest negative subnormal (0x81 = -2^-10) pulled three quarters of the way to zero by weight decay alone:
    # the sum -2^-12 rounds to a zero that keeps its sign only where the format has a negative zero
    out, _, _ = oracle.qat_adamw_step_format8(np.array([0x81], np.uint8), z[:1], z[:1], z[:1], d, (0.75, 0.9, 0.999, 1e-8, 1.0, 0.1, 0.001), RNE, 0, 0, 1)
    assert list(out) == [0x00]
    out, _, _ = oracle.qat_adamw_step_format8(np.array([0x81], np.uint8), z[:1], z[:1], z[:1], E4M3, (0.75, 0.9, 0.999, 1e-8, 1.0, 0.1, 0.001), RNE, 0, 0, 1)
    assert list(out) == [0x80]


# --------------------------------------------- binary8p4 as a target id of the fixed-format entries ----
P4 = 3


def test_binary8p4_target_id_follows_its_descriptor(oracle):
    """Target id 3 (P3109 binary8p4) of round / round_from16 / block-scaled / QAT / statistics is the generic rule
    under the binary8p4 descriptor: same codes as the descriptor entry points, same decode, ulp from Eq. (2)."""
    rng = np.random.default_rng(12)
    x = np.concatenate([rng.integers(0, 1 << 32, 3000, dtype=np.uint32).view(np.float32), inputs_below_max(rng, BINARY8P4, 3000),
                        np.array([224.0, 232.0, np.nextafter(np.float32(232.0), np.float32(np.inf)), np.inf, -np.inf, np.nan, -0.0, -2.0 ** -20], dtype=np.float32)])
    for variant, nbits in ((RNE, 0), (SRFF, 3), (SRF, 2), (SRC, 4), (SRC, 16)):
        for xv in x[::3]:
            n = int(rng.integers(0, 1 << max(nbits, 1)))
            assert oracle.round_with_n(xv, P4, variant, max(nbits, 1), n) == oracle.round_format8_with_n(xv, BINARY8P4, variant, max(nbits, 1), n)
        assert np.array_equal(oracle.round_(x, P4, variant, nbits, seed=4, offset=9), oracle.round_format8(x, FROM_FP32, BINARY8P4, variant, nbits, 4, 9))
        x16 = rng.integers(0, 1 << 16, 4000, dtype=np.uint16)
        for src in (FROM_BF16, FROM_FP16):
            assert np.array_equal(oracle.round_from16(x16, src, P4, variant, nbits, seed=4, offset=9),
                                  oracle.round_format8(x16, src, BINARY8P4, variant, nbits, 4, 9))
    for code in range(256):
        a, b = oracle.decode(code, P4), oracle.decode_format8(code, BINARY8P4)
        assert (math.isnan(a) and math.isnan(b)) or a == b
    assert oracle.ulp(1.0, P4) == 0.125 and oracle.ulp(2.0 ** -9, P4) == 2.0 ** -10 and oracle.ulp(200.0, P4) == 16.0
    # QAT: the fixed-id step equals the descriptor step
    n = 4000
    w8 = rng.integers(0, 256, n).astype(np.uint8)
    g16, m16, v16 = _bf16_codes(rng.standard_normal(n) * 0.3), _bf16_codes(rng.standard_normal(n) * 0.05), _bf16_codes(rng.random(n) * 0.02)
    params = (1e-2, 0.9, 0.999, 1e-8, 0.01, 0.1, 0.001)
    for variant, nbits in ((RNE, 0), (SRFF, 3), (SRC, 3)):
        a = oracle.qat_adamw_step(w8, g16, m16, v16, P4, params, variant, nbits, seed=7, step=5, offset=9)
        b = oracle.qat_adamw_step_format8(w8, g16, m16, v16, BINARY8P4, params, variant, nbits, seed=7, step=5, offset=9)
        assert all(np.array_equal(p, q) for p, q in zip(a, b))
    # block-scaled: emax = 7, elements are the plain rounding of the scaled values, a NaN block is all 0x80
    xb = (rng.standard_normal(32 * 50) * np.exp2(rng.integers(-20, 20, 32 * 50))).astype(np.float32)
    xb[40] = np.nan
    codes, scales = oracle.round_block_scaled(xb, P4, SRC, 3, seed=3, offset=64)
    for b in range(50):
        blk = xb[32 * b:32 * b + 32]
        if b == 1:
            assert scales[b] == 0xFF and np.all(codes[32:64] == 0x80)
            continue
        s = int(scales[b]) - 127
        assert s == math.frexp(float(np.max(np.abs(blk))))[1] - 1 - 7
        want = oracle.round_format8(np.ldexp(blk.astype(np.float64), -s).astype(np.float32), FROM_FP32, BINARY8P4, SRC, 3, 3, 64 + 32 * b)
        assert np.array_equal(codes[32 * b:32 * b + 32], want)
    # statistics: e = (y - x) / ulp with y decoded under the descriptor
    xs = np.abs(x[np.isfinite(x)][:2000])
    xs = xs[xs <= 224.0]
    st, out = oracle.bias_stats(xs, P4, SRF, 3, 5, 0, xs.size, 0, 1, want_out=True)
    y = np.array([oracle.decode_format8(int(c), BINARY8P4) for c in out])
    e = (y - xs.astype(np.float64)) / np.array([oracle.ulp(v, P4) for v in xs])
    assert st[0, 0] == xs.size and abs(st[0, 1] - y.sum()) <= 1e-9 * abs(y.sum()) and abs(st[0, 2] - e.sum()) < 1e-9 and abs(st[0, 3] - (e * e).sum()) < 1e-9
