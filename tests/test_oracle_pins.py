"""Pins for the CPU oracle: everything here checks oracle/ against facts fixed by the paper
(arXiv 2504.20634) or by mathematics, never against the GPU library.  CPU only."""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from conftest import GOLDEN
from exact_model import (FORMATS, MAX_FINITE, code_value, delta_of, expected_ups, f32_fraction,
                         finite_table, neighbours, pow2)

BF16, E4M3, E5M2 = 0, 1, 2
RNE, SRFF, SRF, SRC = 0, 1, 2, 3
SR_VARIANTS = (SRFF, SRF, SRC)
ALL_FMTS = (BF16, E4M3, E5M2)
DROPPED = {BF16: 16, E4M3: 20, E5M2: 21}      # D = 24 - P for fp32 inputs in the target-normal range


def _f32(bits):
    return np.array(bits, dtype=np.uint32).view(np.float32)


def _rand_inputs(rng, fmt, count):
    """fp32 values spread over the whole finite range of fmt, target subnormals included."""
    name = FORMATS[fmt][0]
    lo, hi = {"bf16": (0, 254), "e4m3": (127 - 14, 127 + 8), "e5m2": (127 - 22, 127 + 15)}[name]
    bits = rng.integers(0, 1 << 32, size=count, dtype=np.uint32)
    field = rng.integers(lo, hi + 1, size=count, dtype=np.uint32)
    x = ((bits & np.uint32(0x007FFFFF)) | (field << np.uint32(23))).view(np.float32)
    M = float(MAX_FINITE[fmt])
    return x[np.abs(x.astype(np.float64)) <= M]


# ------------------------------------------------------------------ Philox -----------------
def test_philox_known_answers(oracle):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(t, 16) for t in r]
        got = oracle.philox4x32_10(v[0:4], v[4:6])
        assert [int(g) for g in got] == v[6:10]


@pytest.mark.parametrize("nbits", [1, 2, 3, 4, 5, 6, 8, 11, 12, 16, 17, 24])
def test_random_bits_are_slices_of_the_block(oracle, nbits):
    """Convention pin: element i takes the low N bits of slot i mod (128/W) of block i div (128/W),
    W the next power of two >= N; counter = (block, step), key = seed."""
    W = 1
    while W < nbits:
        W *= 2
    per = 128 // W
    seed, step = 0x0123456789ABCDEF, 0x1_0000_0007
    for blk in (0, 1, 5, (1 << 32) + 3):
        words = oracle.philox4x32_10([blk & 0xFFFFFFFF, blk >> 32, step & 0xFFFFFFFF, step >> 32],
                                     [seed & 0xFFFFFFFF, seed >> 32])
        big = sum(int(w) << (32 * k) for k, w in enumerate(words))
        for slot in (0, 1, per // 2, per - 1):
            want = (big >> (slot * W)) & ((1 << nbits) - 1)
            assert oracle.random_bits(seed, step, blk * per + slot, nbits) == want


# ------------------------------------------------------------------ formats ----------------
def test_decode_matches_library_views(oracle):
    """Eq. (1) decode equals the value a library assigns to the same bits."""
    codes = np.arange(65536, dtype=np.uint16)
    ref = torch.from_numpy(codes.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    got = np.array([oracle.decode(int(c), BF16) for c in codes])
    assert np.array_equal(np.isnan(ref), np.isnan(got))
    assert np.array_equal(ref[~np.isnan(ref)], got[~np.isnan(got)])
    for fmt, tdt in ((E4M3, torch.float8_e4m3fn), (E5M2, torch.float8_e5m2)):
        codes = np.arange(256, dtype=np.uint8)
        ref = torch.from_numpy(codes).view(tdt).to(torch.float64).numpy()
        got = np.array([oracle.decode(int(c), fmt) for c in codes])
        assert np.array_equal(np.isnan(ref), np.isnan(got))
        assert np.array_equal(ref[~np.isnan(ref)], got[~np.isnan(got)])


def test_max_finite_and_tables():
    for fmt in ALL_FMTS:
        vals, _ = finite_table(fmt)
        assert vals[-1] == MAX_FINITE[fmt]
    assert len(finite_table(E4M3)[0]) == 127 and len(finite_table(E5M2)[0]) == 124


@pytest.mark.parametrize("fmt,tdt", [(BF16, torch.bfloat16), (E5M2, torch.float8_e5m2),
                                     (E4M3, torch.float8_e4m3fn)])
def test_rne_matches_library_cast(oracle, fmt, tdt):
    """Sec. II-A ties-to-even, and the out-of-range rule (IEEE round to nearest), against the
    platform's own cast.  E4M3 is compared inside the finite range only: this build saturates
    above 448 where the library cast produces NaN."""
    rng = np.random.default_rng(11)
    bits = rng.integers(0, 1 << 32, size=200000, dtype=np.uint32)
    if fmt != BF16:   # concentrate on the target's range, keep some far outside it
        name = FORMATS[fmt][0]
        lo, hi = {"e4m3": (127 - 14, 127 + 10), "e5m2": (127 - 22, 127 + 18)}[name]
        field = rng.integers(lo, hi + 1, size=bits.size, dtype=np.uint32)
        bits = (bits & np.uint32(0x807FFFFF)) | (field << np.uint32(23))
    # exact ties and near-ties in the target's grid
    D = DROPPED[fmt]
    ties = (bits & ~np.uint32((1 << D) - 1)) | np.uint32(1 << (D - 1))
    x = np.concatenate([bits, ties, ties + np.uint32(1), ties - np.uint32(1)]).view(np.float32)
    x = x[~np.isnan(x)]
    if fmt == E4M3:
        x = x[np.abs(x) <= 448.0]
    got = oracle.round_(x, fmt, RNE, 0, seed=0)
    ref_t = torch.from_numpy(x).to(tdt)
    ref = ref_t.view(torch.int16 if fmt == BF16 else torch.uint8).numpy().view(got.dtype)
    assert np.array_equal(got, ref)


def test_specials_and_out_of_range(oracle):
    """Readings for NaN, infinities, zeros and |x| > M (deterministic, Sec. II)."""
    nan, inf = np.float32(np.nan), np.float32(np.inf)
    for variant, nbits in ((RNE, 0), (SRFF, 2), (SRF, 3), (SRC, 8)):
        for n in (0, (1 << max(nbits, 1)) - 1):
            r = lambda x, fmt: oracle.round_with_n(x, fmt, variant, max(nbits, 1), n)
            # NaN keeps its sign and becomes the canonical quiet NaN
            assert r(nan, BF16) == 0x7FC0 and r(-nan, BF16) == 0xFFC0
            assert r(nan, E4M3) == 0x7F and r(-nan, E4M3) == 0xFF
            assert r(nan, E5M2) == 0x7E and r(-nan, E5M2) == 0xFE
            # zeros keep their sign
            for fmt in ALL_FMTS:
                K = FORMATS[fmt][1]
                assert r(np.float32(0.0), fmt) == 0 and r(np.float32(-0.0), fmt) == 1 << (K - 1)
            # infinities
            assert r(inf, BF16) == 0x7F80 and r(-inf, BF16) == 0xFF80
            assert r(inf, E5M2) == 0x7C and r(-inf, E5M2) == 0xFC
            assert r(inf, E4M3) == 0x7E and r(-inf, E4M3) == 0xFE          # saturating format
            # E4M3: everything above 448 saturates, 448 itself is exact
            assert r(np.float32(448.0), E4M3) == 0x7E
            assert r(np.float32(449.0), E4M3) == 0x7E and r(np.float32(-1e30), E4M3) == 0xFE
            # E5M2: M = 57344 = 0x7B; halfway to the next grid point (61440) and beyond -> inf
            assert r(np.float32(57344.0), E5M2) == 0x7B
            assert r(np.float32(61439.0), E5M2) == 0x7B
            assert r(np.float32(61440.0), E5M2) == 0x7C and r(np.float32(-1e9), E5M2) == 0xFC
            # bf16: M = 0x7F7F0000; below the midpoint 0x7F7F8000 -> M, at or above -> inf
            assert r(_f32(0x7F7F0000), BF16) == 0x7F7F
            assert r(_f32(0x7F7F7FFF), BF16) == 0x7F7F
            assert r(_f32(0x7F7F8000), BF16) == 0x7F80
            assert r(_f32(0xFF7FFFFF), BF16) == 0xFF80


# ------------------------------------------------------------------ structure --------------
@pytest.mark.parametrize("fmt", ALL_FMTS)
def test_result_is_a_bracketing_neighbour_and_representables_are_fixed(oracle, fmt):
    """Eq. (5): sigma is floor or floor+1, so the result is one of the two neighbours; and
    delta = 0 never rounds up because n 2^-N < 1 and (n + 1/2) 2^-N < 1 (Sec. II-B)."""
    rng = np.random.default_rng(21 + fmt)
    K = FORMATS[fmt][1]
    xs = _rand_inputs(rng, fmt, 1500)
    # add every representable value (both signs) of the 8-bit formats / a sample of bf16 codes
    vals, codes = finite_table(fmt)
    take = range(len(vals)) if fmt != BF16 else rng.integers(0, len(vals), 400)
    rep = np.array([float(vals[i]) for i in take], dtype=np.float32)
    for nbits in (1, 2, 3, 8, 16):
        for variant in SR_VARIANTS:
            for x in np.concatenate([xs[:300], -xs[300:400]]):
                n = int(rng.integers(0, 1 << nbits))
                code = oracle.round_with_n(x, fmt, variant, nbits, n)
                lo, hi = neighbours(abs(f32_fraction(x)), fmt)
                sign = (1 << (K - 1)) if np.signbit(x) else 0
                assert code in (sign | lo, sign | hi), (float(x), fmt, variant, nbits, n, hex(code))
            for x in rep[:: max(1, len(rep) // 120)]:
                lo, hi = neighbours(f32_fraction(x), fmt)
                assert lo == hi
                for n in (0, 1, (1 << nbits) - 1):
                    assert oracle.round_with_n(x, fmt, variant, nbits, n) == lo
                    assert oracle.round_with_n(-x, fmt, variant, nbits, n) == (lo | (1 << (K - 1)))


@pytest.mark.parametrize("fmt", ALL_FMTS)
@pytest.mark.parametrize("nbits", [1, 2, 3, 4, 6, 8, 12])
def test_exhaustive_round_up_counts(oracle, fmt, nbits):
    """Enumerating all 2^N draws: the number that round up equals the count implied by each
    predicate (Sec. II-B, Eq. (7)), for inputs over the whole range incl. target subnormals."""
    rng = np.random.default_rng(100 * fmt + nbits)
    xs = _rand_inputs(rng, fmt, 400)
    # force ties / near ties of the inner Round of SRC: delta 2^N exactly half-integral
    D = DROPPED[fmt]
    base = xs[:64].view(np.uint32) & ~np.uint32((1 << D) - 1)
    if D - nbits - 1 >= 0:
        ties = base | (rng.integers(0, 1 << nbits, 64).astype(np.uint32) << np.uint32(D - nbits)) \
            | np.uint32(1 << (D - nbits - 1))
        xs = np.concatenate([xs, ties.view(np.float32), (ties + np.uint32(1)).view(np.float32)])
    xs = xs[np.abs(xs.astype(np.float64)) <= float(MAX_FINITE[fmt])]
    for variant in SR_VARIANTS:
        ups = oracle.count_up(xs, fmt, variant, nbits)
        for x, u in zip(xs, ups):
            _, delta = delta_of(abs(f32_fraction(x)), fmt)
            assert int(u) == expected_ups(delta, variant, nbits), (float(x), variant, nbits)


@pytest.mark.parametrize("fmt,nbits", [(E4M3, 19), (E4M3, 24), (E5M2, 23)])
def test_exhaustive_round_up_counts_many_bits_below_the_smallest_normal(oracle, fmt, nbits):
    """All 2^N draws for N up to 24 on inputs in and far below the target's subnormal range, where the fixed grid
    (Eq. (2) clamps the exponent) drops more than 24 bits: the counts still equal those the predicates imply, in
    exact rational arithmetic."""
    rng = np.random.default_rng(5 * fmt + nbits)
    lo_field = {E4M3: 127 - 9 - 30, E5M2: 127 - 16 - 30}[fmt]                 # down to 2^-30 of the subnormal spacing
    hi_field = {E4M3: 127 - 6, E5M2: 127 - 14}[fmt]                           # the smallest normal binade
    fields = rng.integers(lo_field, hi_field + 1, 5).astype(np.uint32)
    xs = ((fields << np.uint32(23)) | rng.integers(0, 1 << 23, 5, dtype=np.uint32)).view(np.float32)
    xs = np.concatenate([xs, np.array([2.0 ** -9 * 1.5, 2.0 ** -16 * 2.5 + 2.0 ** -39], dtype=np.float32)])   # a tie, a near tie
    for variant in SR_VARIANTS:
        ups = oracle.count_up(xs, fmt, variant, nbits)
        for x, u in zip(xs, ups):
            _, delta = delta_of(abs(f32_fraction(x)), fmt)
            assert int(u) == expected_ups(delta, variant, nbits), (float(x), variant, nbits)


@pytest.mark.parametrize("fmt,nbits", [(BF16, 16), (BF16, 18), (E4M3, 20), (E5M2, 21), (E5M2, 22)])
def test_enough_bits_is_exact_sr(oracle, fmt, nbits):
    """N >= D: every variant rounds up with probability exactly delta (App. A-C: the floor
    in the SRFF sum disappears and the bias is zero)."""
    D = DROPPED[fmt]
    name = FORMATS[fmt][0]
    one = {"bf16": 127, "e4m3": 127, "e5m2": 127}[name] << 23          # the binade [1,2)
    rng = np.random.default_rng(7)
    frac = rng.integers(0, 1 << 23, 3, dtype=np.uint32)
    xs = (np.uint32(one) | frac).view(np.float32)
    for variant in SR_VARIANTS:
        ups = oracle.count_up(xs, fmt, variant, nbits)
        for x, u in zip(xs, ups):
            _, delta = delta_of(f32_fraction(x), fmt)
            assert Fraction(int(u), 1 << nbits) == delta


# ------------------------------------------------------------------ closed-form biases -----
def _grid_bias(oracle, fmt, variant, nbits, start_bits, count, stride_bits=1):
    """Exact mean over the grid of E_n[up] - delta, for `count` inputs start + k*stride (bit
    patterns) that tile whole target intervals."""
    xs = (np.uint32(start_bits) + np.arange(count, dtype=np.uint32) * np.uint32(stride_bits)).view(np.float32)
    ups = oracle.count_up(xs, fmt, variant, nbits)
    total = Fraction(0)
    for x, u in zip(xs, ups):
        _, delta = delta_of(f32_fraction(x), fmt)
        total += Fraction(int(u), 1 << nbits) - delta
    return total / count


@pytest.mark.parametrize("nbits", [1, 2, 3, 4, 8])
def test_closed_form_bias_fp32_to_bf16(oracle, nbits):
    """All 2^16 fp32 values of one bf16 interval [1, 1 + 2^-7): D = 16 excess bits.
    SRFF (2^-D - 2^-N)/2, SRF +2^-(D+1), SRC 0 (Sec. III-E, III-F; App. A-C, A-D).  At N = 2
    SRFF gives -0.12499..., the -0.124 ~ -2^-3 printed under Fig. 1."""
    D = 16
    xs = (np.uint32(0x3F800000) + np.arange(1 << D, dtype=np.uint32)).view(np.float32)
    i = np.arange(1 << D, dtype=object)
    for variant, want in ((SRFF, (pow2(-D) - pow2(-nbits)) / 2), (SRF, pow2(-(D + 1))), (SRC, 0)):
        ups = oracle.count_up(xs, BF16, variant, nbits)
        got = Fraction(int(ups.astype(object).sum()), (1 << nbits) << D) - Fraction(int(i.sum()), 1 << (2 * D))
        assert got == want, (variant, nbits, float(got))
    if nbits == 2:
        printed = -0.124      # tests/golden/paper_bias_values.txt, fig1 srff
        assert abs(float((pow2(-D) - pow2(-2)) / 2) - printed) < 1.5e-3


@pytest.mark.parametrize("fmt,D,start", [(E4M3, 20, 0x3F800000), (E5M2, 21, 0x40000000)])
def test_closed_form_bias_fp32_to_fp8_interval(oracle, fmt, D, start):
    """One full target interval of an fp8 format (2^D fp32 inputs), N = 2 and 3."""
    for nbits in (2, 3):
        for variant, want in ((SRFF, (pow2(-D) - pow2(-nbits)) / 2), (SRF, pow2(-(D + 1))), (SRC, 0)):
            xs = (np.uint32(start) + np.arange(1 << D, dtype=np.uint32)).view(np.float32)
            ups = oracle.count_up(xs, fmt, variant, nbits)
            s_ups = int(ups.astype(np.int64).sum())
            s_delta = Fraction((1 << D) * ((1 << D) - 1) // 2, 1 << D)
            got = (Fraction(s_ups, 1 << nbits) - s_delta) / (1 << D)
            assert got == want, (fmt, variant, nbits, float(got))


def test_fig2_printed_biases(oracle):
    """Fig. 2: bf16-valued inputs rounded to a precision-3 target (D = 5 excess bits).  The
    printed -0.046875 / +0.015625 / 0.000 are reproduced exactly at N = 3."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "paper_bias_values.txt"))
            if l.strip() and not l.startswith("#")]
    fig2 = {r[1]: (int(r[2]), int(r[3]), Fraction(r[4])) for r in rows if r[0] == "fig2"}
    names = {SRFF: "srff", SRF: "srf", SRC: "src"}
    # all 32 bf16 values of the E5M2 interval [2, 2.5): fp32 patterns 0x40000000 + k * 2^16
    for variant in SR_VARIANTS:
        nbits, D, want = fig2[names[variant]]
        assert D == 5
        got = _grid_bias(oracle, E5M2, variant, nbits, 0x40000000, 1 << D, stride_bits=1 << 16)
        assert got == want, (variant, float(got))
    # with the caption's "2 bits" the SRFF value would be -0.109375, not the printed one
    assert _grid_bias(oracle, E5M2, SRFF, 2, 0x40000000, 32, 1 << 16) == Fraction(-7, 64)


@pytest.mark.parametrize("D,stride,fmt,start", [(5, 1 << 16, E5M2, 0x40800000), (4, 1 << 16, E4M3, 0x3F000000),
                                                (6, 1 << 10, BF16, 0x3F800000)])
def test_exact_floor_forms_any_n(oracle, D, stride, fmt, start):
    """App. A-C / A-D final sums, valid for any N and D:
       SRFF: 2^-N sum_n 2^-D floor(2^(D-N) n)           - (1 - 2^-D)/2
       SRF : 2^-N sum_n 2^-D floor(n 2^(D-N) + 2^(D-N-1)) - (1 - 2^-D)/2
    including N > D where they reach zero; SRC is zero throughout."""
    for nbits in range(1, 9):
        srff = sum(Fraction(int(pow2(D - nbits) * n // 1), 1 << D) for n in range(1 << nbits)) / (1 << nbits) \
            - (1 - pow2(-D)) / 2
        srf = sum(Fraction(int((pow2(D - nbits) * n + pow2(D - nbits - 1)) // 1), 1 << D)
                  for n in range(1 << nbits)) / (1 << nbits) - (1 - pow2(-D)) / 2
        assert _grid_bias(oracle, fmt, SRFF, nbits, start, 1 << D, stride) == srff
        assert _grid_bias(oracle, fmt, SRF, nbits, start, 1 << D, stride) == srf
        assert _grid_bias(oracle, fmt, SRC, nbits, start, 1 << D, stride) == 0
        if nbits >= D:
            assert srff == 0
        if nbits <= D:
            assert srff == (pow2(-D) - pow2(-nbits)) / 2
        if nbits < D:
            assert srf == pow2(-(D + 1))


def test_src_ties_go_to_even(oracle):
    """Eq. (7) with Round = nearest, ties to even: delta 2^N = k + 1/2 rounds to the even one of
    k, k+1, so exactly that many draws round up."""
    N = 2
    for k in range(4):
        # bf16 interval [1, 1+2^-7): delta = (k + 1/2)/4  -> fp32 offset (2k+1) * 2^13 ulps
        x = _f32(0x3F800000 + (2 * k + 1) * (1 << 13))
        ups = int(oracle.count_up(np.array([x]), BF16, SRC, N)[0])
        assert ups == (k if k % 2 == 0 else k + 1)


# ------------------------------------------------------------------ sampled behaviour ------
def test_fig1_sampled_bias(oracle):
    """Fig. 1's experiment with this build's bit source on the benchmark's grid: 1024 X values
    evenly spaced over 16 bf16 ulps (a 2^-6-ulp lattice, i.e. D = 6 excess bits), 5000 samples
    each, N = 2.  The sampled mean bias must sit on the finite-precision closed forms of
    Sec. III-E at D = 6 -- SRFF (2^-6 - 2^-2)/2 = -0.1171875, SRF 2^-7, SRC 0 -- within the
    noise of the draws (sigma ~ 0.43 / sqrt(5.12e6) ~ 2e-4 ulp), and SRFF's per-X means lie
    below Y = X (caption of Fig. 1, left)."""
    from paper_2504_20634_amd import workloads
    x, X = workloads.fig1_grid(points=1024, samples=5000)
    for variant, want in ((SRFF, -0.1171875), (SRF, 0.0078125), (SRC, 0.0)):
        stats, _ = oracle.bias_stats(x, BF16, variant, 2, seed=0, offset=0, group=5000, first_bin=0,
                                     nbins=1024)
        assert np.all(stats[:, 0] == 5000)
        bias = stats[:, 2].sum() / stats[:, 0].sum()
        assert abs(bias - want) < 1e-3, (variant, bias)
        if variant == SRFF:
            below = stats[:, 1] / 5000 <= X.astype(np.float64)
            assert below.mean() > 0.9   # X with delta a multiple of 1/4 are individually unbiased


def test_chunked_calls_equal_whole(oracle):
    from paper_2504_20634_amd import workloads
    x = workloads.scaled_normal(5000, seed=9)
    for fmt in ALL_FMTS:
        for variant, nbits in ((SRFF, 1), (SRF, 3), (SRC, 6), (SRFF, 16)):
            whole = oracle.round_(x, fmt, variant, nbits, seed=4, offset=77)
            parts = [oracle.round_(x[a:b], fmt, variant, nbits, seed=4, offset=77 + a)
                     for a, b in ((0, 1), (1, 130), (130, 4099), (4099, 5000))]
            assert np.array_equal(whole, np.concatenate(parts))
            assert np.array_equal(whole, oracle.round_(x, fmt, variant, nbits, 4, 77, nthreads=3))


def test_stats_sum_is_the_exact_integer_sum(oracle):
    """sum e from the fp64 accumulation equals the integer sum of (code << 16) - bits(x),
    scaled by 2^-16, for bf16 in the normal range (no rounding can occur in that sum)."""
    rng = np.random.default_rng(3)
    x = (1.0 + rng.random(40000)).astype(np.float32)
    for variant in SR_VARIANTS:
        stats, out = oracle.bias_stats(x, BF16, variant, 4, seed=5, offset=1000, group=10000,
                                       first_bin=0, nbins=5, want_out=True)
        diff = (out.astype(np.int64) << 16) - x.view(np.uint32).astype(np.int64)
        bins = (1000 + np.arange(x.size)) // 10000
        for b in range(5):
            assert stats[b, 0] == np.sum(bins == b)
            assert stats[b, 2] == float(diff[bins == b].sum()) / 65536.0
            y = (out[bins == b].astype(np.uint32) << 16).view(np.float32).astype(np.float64)
            assert abs(stats[b, 1] - y.sum()) <= 1e-12 * abs(y.sum())
            assert abs(stats[b, 3] - np.sum((diff[bins == b] / 65536.0) ** 2)) <= 1e-9 * stats[b, 3]


@pytest.mark.parametrize("fmt", [E4M3, E5M2])
def test_stats_sums_are_the_exact_rational_sums(oracle, fmt):
    """Per-bin {count, sum y, sum e, sum e^2} against sums of exact rationals: y from Eq. (1) on the
    returned code, ulp_t(x) = 2^(max(floor(log2 |x|), 1 - B) - P + 1) from Eq. (2) with integer
    arithmetic on x's own fraction, e = (y - x) / ulp_t(x).  Inputs cover the target's normal range,
    its subnormal range, values far below the smallest subnormal, both signs, zero, and (E4M3) the
    saturated range above M, where y = +-M.  sum e is a sum of multiples of one power of two that
    fits fp64, so the oracle's fp64 accumulation must reproduce it exactly."""
    _, K, P, B, has_inf = FORMATS[fmt]
    rng = np.random.default_rng(40 + fmt)
    group = 500
    M = float(MAX_FINITE[fmt])
    parts = [rng.uniform(2.0 ** (1 - B), M, group),                                        # normal range
             rng.uniform(2.0 ** (2 - B - P), 2.0 ** (1 - B), group),                        # subnormal range
             rng.uniform(2.0 ** (-B - P - 20), 2.0 ** (2 - B - P), group),                  # below the smallest subnormal
             -np.exp(rng.uniform(np.log(2.0 ** (-B - P - 3)), np.log(M), group)),           # negative, every range
             np.concatenate([np.zeros(5), -np.zeros(5), rng.uniform(2.0 ** -B, 2.0 ** (3 - B), group - 10)])]
    if not has_inf:
        parts.append(rng.uniform(M, 8 * M, group) * np.where(rng.integers(0, 2, group) == 1, -1.0, 1.0))   # saturates to +-M
    x = np.concatenate(parts).astype(np.float32)
    nbins = len(parts)
    for variant, nbits in ((SRFF, 2), (SRF, 3), (SRC, 3), (RNE, 0), (SRC, 8)):
        stats, out = oracle.bias_stats(x, fmt, variant, nbits, seed=6, offset=0, group=group, first_bin=0, nbins=nbins,
                                       want_out=True)
        for b in range(nbins):
            sy = se = see = Fraction(0)
            for j in range(b * group, (b + 1) * group):
                xf = f32_fraction(x[j])
                code = int(out[j])
                mag = code_value(code & ((1 << (K - 1)) - 1), fmt)
                assert mag is not None
                y = -mag if code >> (K - 1) else mag
                a = abs(xf)
                lg = (a.numerator.bit_length() - a.denominator.bit_length()) if a else 1 - B
                if a and Fraction(2) ** lg > a:
                    lg -= 1
                ulp = Fraction(2) ** (max(lg, 1 - B) - P + 1)
                e = (y - xf) / ulp
                sy += y
                se += e
                see += e * e
            assert stats[b, 0] == group
            assert stats[b, 1] == float(sy) or abs(stats[b, 1] - float(sy)) <= 1e-13 * abs(float(sy)), (fmt, variant, b)
            if b < 2 or b >= 4:      # multiples of 2^-(24-P) (2^-24 in the saturated range) below 2^53 of them: exact
                assert stats[b, 2] == float(se), (fmt, variant, nbits, b, stats[b, 2], float(se))
            else:                    # deep inputs: single errors carry more than 53 bits, fp64 rounds each of them
                assert abs(stats[b, 2] - float(se)) <= 1e-12 * max(abs(float(se)), 1.0), (fmt, variant, nbits, b)
            assert abs(stats[b, 3] - float(see)) <= 1e-12 * float(see) + 1e-300, (fmt, variant, nbits, b)


def test_sgd_small_updates(oracle):
    """Updates far below one ulp (Sec. IV: nearest-even stagnates, SRFF drifts): RNE, SRF and
    SRC leave the weights alone; SRFF loses 2^-(N+1) ulp of |w| per step on average, because the
    half of the updates that point toward zero each drop a full ulp with probability 2^-N
    (App. A-A), while the signed mean stays put."""
    from paper_2504_20634_amd import workloads
    n, steps, lr = 4000, 100, 1e-3
    w0 = workloads.sgd_weights(n, seed=3)
    w0 = np.where((w0 & 0x7FFF) < 0x3C00, w0 | 0x3C00, w0).astype(np.uint16)    # keep |w| >= 2^-7
    val = lambda w: (w.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    ulp = np.array([oracle.ulp(v, BF16) for v in val(w0).astype(np.float32)])
    for variant, nbits in ((RNE, 0), (SRF, 2), (SRC, 2), (SRFF, 2), (SRFF, 4)):
        w = w0.copy()
        for t in range(steps):
            g = workloads.sgd_grads(n, t, seed=3, std=1e-3)       # |lr g| ~ 1e-6 << ulp >= 6e-5
            w = oracle.sgd_update(w, g, lr, variant, nbits, seed=8, step=t)
        moved = np.mean((np.abs(val(w)) - np.abs(val(w0))) / ulp) / steps
        if variant == SRFF:
            assert abs(moved + 2.0 ** -(nbits + 1)) < 0.15 * 2.0 ** -(nbits + 1), (nbits, moved)
            assert abs(np.mean(val(w)) - np.mean(val(w0))) < 5e-3
        else:
            assert np.array_equal(w, w0), variant


def test_sgd_is_one_fma_then_round(oracle):
    """The update is a single-rounding fp32 fused multiply-add followed by the bf16 rounding."""
    rng = np.random.default_rng(12)
    # |w| in [1,2), |lr g| in [0.37, 1.48): the exact sum fits in a double, so the fp64 value
    # below is exact and its cast to fp32 is the single rounding of a fused multiply-add
    w = (rng.integers(0x3F80, 0x4000, 3000).astype(np.uint16)
         | (rng.integers(0, 2, 3000).astype(np.uint16) << 15)).astype(np.uint16)
    g = (rng.uniform(1.0, 4.0, w.size) * rng.choice([-1.0, 1.0], w.size)).astype(np.float32)
    lr = np.float32(0.37)
    wf = (w.astype(np.uint32) << 16).view(np.float32)
    x = (wf.astype(np.float64) - np.float64(lr) * g.astype(np.float64)).astype(np.float32)
    for variant, nbits in ((RNE, 0), (SRFF, 3), (SRC, 5)):
        got = oracle.sgd_update(w, g, lr, variant, nbits, seed=2, step=6, offset=10)
        want = np.array([oracle.round_with_n(xi, BF16, variant, max(nbits, 1),
                                             oracle.random_bits(2, 6, 10 + j, nbits) if variant else 0)
                         for j, xi in enumerate(x)], dtype=np.uint16)
        assert np.array_equal(got, want)


# ------------------------------------------------------------------ narrow sources ---------
SRC_BF16, SRC_FP16 = 0, 1


@pytest.mark.parametrize("src,tdt", [(SRC_BF16, torch.bfloat16), (SRC_FP16, torch.float16)])
def test_widening_matches_library(oracle, src, tdt):
    """Eq. (1) on all 65536 source codes equals the library's widening to fp32 (NaNs: sign and
    NaN-ness agree)."""
    codes = np.arange(65536, dtype=np.uint16)
    ref = torch.from_numpy(codes.view(np.int16)).view(tdt).to(torch.float32).numpy().view(np.uint32)
    got = np.array([oracle.widen16(int(c), src) for c in codes], dtype=np.uint32)
    nan = np.isnan(ref.view(np.float32))
    assert np.array_equal(ref[~nan], got[~nan])
    assert np.all(np.isnan(got[nan].view(np.float32))) and np.array_equal(ref[nan] >> 31, got[nan] >> 31)


def test_narrow_source_is_widen_then_round(oracle):
    rng = np.random.default_rng(4)
    codes = rng.integers(0, 1 << 16, 20000, dtype=np.uint16)
    for src, tdt in ((SRC_BF16, torch.bfloat16), (SRC_FP16, torch.float16)):
        wide = torch.from_numpy(codes.view(np.int16)).view(tdt).to(torch.float32).numpy()
        for fmt in (E4M3, E5M2):
            for variant, nbits in ((RNE, 0), (SRFF, 2), (SRF, 3), (SRC, 4), (SRFF, 9)):
                a = oracle.round_from16(codes, src, fmt, variant, nbits, seed=6, offset=123)
                b = oracle.round_(wide, fmt, variant, nbits, seed=6, offset=123)
                assert np.array_equal(a, b)


@pytest.mark.parametrize("src,fmt,D,start16", [(SRC_BF16, E4M3, 4, 0x3F80), (SRC_BF16, E5M2, 5, 0x4000),
                                               (SRC_FP16, E4M3, 7, 0x3C00), (SRC_FP16, E5M2, 8, 0x4000)])
def test_narrow_source_closed_forms(oracle, src, fmt, D, start16):
    """Sec. III-E with the source formats the paper names: all 2^D source values of one target
    interval, all 2^N draws.  SRFF (2^-D - 2^-N)/2 for N <= D (0 beyond), SRF 2^-(D+1) for N < D,
    SRC 0.  bf16 -> E5M2 at N = 3 is Fig. 2's setting."""
    codes = (start16 + np.arange(1 << D)).astype(np.uint16)
    wide = np.array([oracle.widen16(int(c), src) for c in codes], dtype=np.uint32).view(np.float32)
    for nbits in (1, 2, 3, 4, 6):
        for variant in SR_VARIANTS:
            ups = oracle.count_up(wide, fmt, variant, nbits)
            total = Fraction(0)
            for x, u in zip(wide, ups):
                _, delta = delta_of(f32_fraction(x), fmt)
                total += Fraction(int(u), 1 << nbits) - delta
            got = total / (1 << D)
            if variant == SRFF:
                want = (pow2(-D) - pow2(-nbits)) / 2 if nbits <= D else 0
            elif variant == SRF:
                want = pow2(-(D + 1)) if nbits < D else None
            else:
                want = 0
            if want is not None:
                assert got == want, (src, fmt, variant, nbits, float(got))


# ------------------------------------------------------------------ fused QAT step (Alg. 1) ----
def _bf16_codes(a):
    """fp32 array -> bf16 codes by the library's round-to-nearest-even cast."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def _bf16_values(c):
    return (c.astype(np.uint32) << 16).view(np.float32)


def _fp8_values(codes, fmt):
    tdt = torch.float8_e4m3fn if fmt == E4M3 else torch.float8_e5m2
    return torch.from_numpy(codes).view(tdt).to(torch.float32).numpy()


@pytest.mark.parametrize("hyper", [(3e-2, 0.9, 0.95, 1e-8, 0.1), (0.1, 0.8, 0.9, 1e-6, 5.0)],
                         ids=["small_decay", "large_decay"])
@pytest.mark.parametrize("fmt", [E4M3, E5M2])
def test_qat_step_tracks_library_adamw(oracle, fmt, hyper):
    """Three steps of Alg. 1 with the oracle against torch.optim.AdamW in fp32 on the same gradients:
    the bf16 moments stay within bf16 rounding of the fp32 moments, and each new 8-bit weight is within
    one target ulp (plus the 16-bit roundings) of the fp32 update of the previous 8-bit weight.  A
    dropped term, a wrong sign or a missing bias correction moves results by far more."""
    rng = np.random.default_rng(17)
    n = 4000
    vals, codes = finite_table(fmt)
    pick = rng.integers(8, len(codes) - 8, n)
    w8 = (np.array(codes, dtype=np.uint8)[pick] | (rng.integers(0, 2, n).astype(np.uint8) << 7)).astype(np.uint8)
    lr, b1, b2, eps, wd = hyper      # large_decay: lr * wd = 0.5, so the decay term alone moves weights by many ulps
    m16 = np.zeros(n, np.uint16)
    v16 = np.zeros(n, np.uint16)
    m_ref = np.zeros(n, np.float64)
    v_ref = np.zeros(n, np.float64)
    for t in (1, 2, 3):
        g16 = _bf16_codes(rng.standard_normal(n) * 0.5)
        g = _bf16_values(g16).astype(np.float64)
        w_prev = _fp8_values(w8, fmt).astype(np.float64)
        m_prev, v_prev = m_ref.copy(), v_ref.copy()
        # library step on the current 8-bit weights with its own fp32 state replaced by the references
        p = torch.nn.Parameter(torch.from_numpy(w_prev.astype(np.float32)))
        opt = torch.optim.AdamW([p], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
        p.grad = torch.from_numpy(g.astype(np.float32))
        opt.state[p] = {"step": torch.tensor(float(t - 1)), "exp_avg": torch.from_numpy(m_ref.astype(np.float32)),
                        "exp_avg_sq": torch.from_numpy(v_ref.astype(np.float32))}
        opt.step()
        target = p.detach().numpy().astype(np.float64)
        m_ref = opt.state[p]["exp_avg"].numpy().astype(np.float64)
        v_ref = opt.state[p]["exp_avg_sq"].numpy().astype(np.float64)
        params = (lr, b1, b2, eps, wd, 1 - b1 ** t, 1 - b2 ** t)
        w8, m16, v16 = oracle.qat_adamw_step(w8, g16, m16, v16, fmt, params, SRC, 3, seed=5, step=t)
        m_got, v_got = _bf16_values(m16).astype(np.float64), _bf16_values(v16).astype(np.float64)
        # one bf16 rounding of the result, plus fp32 rounding noise relative to the terms that were added
        m_tol = 2.0 ** -8 * np.abs(m_ref) + 2.0 ** -20 * (np.abs(m_prev) + np.abs(g)) + 1e-40
        v_tol = 2.0 ** -8 * np.abs(v_ref) + 2.0 ** -20 * (np.abs(v_prev) + g * g) + 1e-40
        assert np.all(np.abs(m_got - m_ref) <= m_tol), np.max(np.abs(m_got - m_ref) / m_tol)
        assert np.all(np.abs(v_got - v_ref) <= v_tol), np.max(np.abs(v_got - v_ref) / v_tol)
        w_new = _fp8_values(w8, fmt).astype(np.float64)
        ulp8 = np.array([oracle.ulp(np.float32(x), fmt) for x in target])
        slack = ulp8 + 2.0 ** -6 * np.abs(target) + 2.0 ** -5 * np.abs(target - w_prev)
        assert np.all(np.abs(w_new - target) <= slack), np.max(np.abs(w_new - target) / slack)
        # restart the reference moments from the 16-bit ones so rounding differences do not pile up
        m_ref, v_ref = m_got, v_got


def test_qat_step_adds_eps_outside_the_root(oracle):
    """Where AdamW's eps sits: u = -lr (m / c1) / (sqrt(v / c2) + eps), not sqrt(v / c2 + eps).  With a zero gradient
    and a zero second moment the denominator is eps itself, so the two placements differ by 1 / sqrt(eps); every
    number below is a power of two, the library's fp32 step is exact and lands on E4M3 values, and the oracle must
    return exactly those (a representable sum is a fixed point of every variant)."""
    lr, b1, b2, eps, wd = 0.125, 0.5, 0.75, 2.0 ** -4, 0.0
    w = np.array([1.0, -1.0, 2.0, 0.5, 4.0, -8.0], dtype=np.float32)
    m = np.array([0.25, -0.25, 0.125, 0.5, -0.5, 0.5], dtype=np.float32)
    p = torch.nn.Parameter(torch.from_numpy(w.copy()))
    opt = torch.optim.AdamW([p], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
    p.grad = torch.zeros(w.size)
    opt.state[p] = {"step": torch.tensor(0.0), "exp_avg": torch.from_numpy(m.copy()), "exp_avg_sq": torch.zeros(w.size)}
    opt.step()
    target = p.detach().numpy()
    # the library's own numbers: m <- m / 2, denominator eps, step lr / c1 * m' / eps = m * 2
    assert np.array_equal(target, w - 2.0 * m)
    vals, codes = finite_table(E4M3)
    lookup = {float(v): c for v, c in zip(vals, codes)}
    w8 = np.array([lookup[abs(float(v))] | (0x80 if v < 0 else 0) for v in w], dtype=np.uint8)
    want8 = np.array([lookup[abs(float(v))] | (0x80 if v < 0 else 0) for v in target], dtype=np.uint8)
    g16 = np.zeros(w.size, np.uint16)
    for variant, nbits in ((RNE, 0), (SRFF, 3), (SRF, 3), (SRC, 3)):
        got, m16, v16 = oracle.qat_adamw_step(w8, g16, _bf16_codes(m), np.zeros(w.size, np.uint16), E4M3,
                                             (lr, b1, b2, eps, wd, 1 - b1, 1 - b2), variant, nbits, seed=3, step=1)
        assert np.array_equal(got, want8), (variant, got, want8)
        assert np.array_equal(_bf16_values(m16), m * np.float32(0.5)) and not v16.any()


def test_qat_step_structure(oracle):
    """lr = 0 leaves every weight where it is (representable values are fixed points of all
    variants); the 8-bit rounding is exactly the narrow-source FBSR of the bf16 sum with the bits of
    (seed, step, index); nearest-even stagnates on tiny updates while the stochastic variants move
    (Sec. IV: "further gradient updates make no change to the weights")."""
    rng = np.random.default_rng(3)
    n = 3000
    for fmt in (E4M3, E5M2):
        vals, codes = finite_table(fmt)
        w8 = (np.array(codes, dtype=np.uint8)[rng.integers(4, len(codes) - 4, n)]
              | (rng.integers(0, 2, n).astype(np.uint8) << 7)).astype(np.uint8)
        g16 = _bf16_codes(rng.standard_normal(n))
        m16 = _bf16_codes(rng.standard_normal(n) * 0.1)
        v16 = _bf16_codes(rng.random(n) * 0.1)
        for variant, nbits in ((RNE, 0), (SRFF, 3), (SRF, 3), (SRC, 3)):
            same, m_a, v_a = oracle.qat_adamw_step(w8, g16, m16, v16, fmt, (0.0, 0.9, 0.999, 1e-8, 0.01, 0.1, 0.001),
                                                   variant, nbits, seed=1, step=4)
            assert np.array_equal(same, w8)
        # the moments do not depend on the variant, the seed or lr
        _, m_b, v_b = oracle.qat_adamw_step(w8, g16, m16, v16, fmt, (0.5, 0.9, 0.999, 1e-8, 0.01, 0.1, 0.001), SRFF, 2, 9, 1)
        assert np.array_equal(m_a, m_b) and np.array_equal(v_a, v_b)
        # tiny updates: |u| far below the spacing of both the 8-bit and the 16-bit grid around w
        params = (1e-6, 0.9, 0.999, 1e-8, 0.0, 0.1, 0.001)
        big = (np.abs(_fp8_values(w8, fmt)) >= 2.0 ** -5)
        stuck, _, _ = oracle.qat_adamw_step(w8, g16, m16, v16, fmt, params, RNE, 0, 1, 1)
        assert np.array_equal(stuck[big], w8[big])
    # the rounding handed to RoundTo8 is the narrow-source one: recompute the bf16 sum in numpy fp32
    fmt, variant, nbits, seed, step, off = E4M3, SRF, 3, 11, 6, 40
    lr, b1, b2, eps, wd, c1, c2 = (np.float32(v) for v in (0.05, 0.9, 0.99, 1e-8, 0.1, 0.3, 0.05))
    w = _fp8_values(w8, fmt)
    g, m0, v0 = _bf16_values(g16), _bf16_values(m16), _bf16_values(v16)
    one = np.float32(1.0)
    fma = lambda a, b, c: (a.astype(np.float64) * b.astype(np.float64) + c.astype(np.float64)).astype(np.float32)
    m1 = fma(np.full(n, b1), m0, (one - b1) * g)
    v1 = fma(np.full(n, b2), v0, (one - b2) * (g * g))
    mq, vq = _bf16_values(_bf16_codes(m1)), _bf16_values(_bf16_codes(v1))
    ratio = (mq / c1) / (np.sqrt(vq / c2) + eps)
    u = -lr * fma(np.full(n, wd), w, ratio)
    s16 = _bf16_codes(w + _bf16_values(_bf16_codes(u)))
    got, _, _ = oracle.qat_adamw_step(w8, g16, m16, v16, fmt, (lr, b1, b2, eps, wd, c1, c2), variant, nbits, seed, step, off)
    want = np.array([oracle.round_with_n(x, fmt, variant, nbits, oracle.random_bits(seed, step, off + j, nbits))
                     for j, x in enumerate(_bf16_values(s16))], dtype=np.uint8)
    assert np.array_equal(got, want)


# ------------------------------------------------------------------ block-scaled targets -------
def test_block_scale_rule_and_composition(oracle):
    """Sec. I-A's scaled tensors with a power-of-two scale per block of 32.  The scale exponent is
    floor(log2 amax) - emax (library frexp), the elements are exactly the plain FBSR of the values
    scaled by that power of two, the block maximum lands in [2^emax, 2^(emax+1)), and multiplying a
    whole tensor by 2^k changes the scale bytes by k and no element code."""
    rng = np.random.default_rng(8)
    n = 32 * 200 + 13                                   # a short last block
    x = (rng.standard_normal(n) * np.exp2(rng.integers(-20, 20, n))).astype(np.float32)
    x[32 * 5:32 * 6] = 0.0                              # a block of zeros
    x[32 * 7 + 3] = np.float32(3.0e38)
    for fmt, emax in ((E4M3, 8), (E5M2, 15)):
        for variant, nbits in ((RNE, 0), (SRFF, 2), (SRF, 3), (SRC, 4)):
            codes, scales = oracle.round_block_scaled(x, fmt, variant, nbits, seed=3, offset=64)
            assert scales.size == (n + 31) // 32
            for b in range(scales.size):
                blk = x[32 * b:32 * b + 32]
                amax = float(np.max(np.abs(blk)))
                if amax == 0.0:
                    assert scales[b] == 0
                    assert not (codes[32 * b:32 * b + 32] & 0x7F).any()
                    continue
                mant, ex = np.frexp(amax)              # amax = mant * 2^ex, mant in [0.5, 1)
                s = max(-127, min(127, int(ex) - 1 - emax))
                assert int(scales[b]) - 127 == s
                scaled = np.ldexp(blk.astype(np.float64), -s)
                assert 2.0 ** emax <= np.max(np.abs(scaled)) < 2.0 ** (emax + 1)
                inexact = scaled.astype(np.float32).astype(np.float64) != scaled
                assert np.all(np.abs(scaled[inexact]) < 2.0 ** -126)      # only fp32 underflow, far below any fp8 grid
                want = oracle.round_(scaled.astype(np.float32), fmt, variant, nbits, seed=3, offset=64 + 32 * b)
                assert np.array_equal(codes[32 * b:32 * b + 32], want)
            for k in (-7, 11):
                xk64 = np.ldexp(x.astype(np.float64), k)
                xk = xk64.astype(np.float32)
                c2, s2 = oracle.round_block_scaled(xk, fmt, variant, nbits, seed=3, offset=64)
                for b in range(scales.size):
                    sl = slice(32 * b, 32 * b + 32)
                    if scales[b] == 0 or not np.array_equal(xk[sl].astype(np.float64), xk64[sl]):
                        continue          # zeros, or the shifted block left fp32's exact range
                    assert np.array_equal(c2[sl], codes[sl]) and int(s2[b]) == int(scales[b]) + k


def test_block_scale_specials(oracle):
    """A block that holds a NaN or an infinity is marked with the scale byte 0xFF and all its elements
    become the positive canonical NaN; neighbouring blocks are untouched.  Scale exponents clamp at
    -127 for blocks of fp32 subnormals."""
    x = np.ones(32 * 4, dtype=np.float32)
    x[40] = np.float32(np.nan)
    x[70] = np.float32(-np.inf)
    x[96:128] = _f32(np.arange(1, 33, dtype=np.uint32))          # fp32 subnormals
    for fmt, nan_code in ((E4M3, 0x7F), (E5M2, 0x7E)):
        codes, scales = oracle.round_block_scaled(x, fmt, SRF, 3, seed=1)
        assert scales[1] == 0xFF and scales[2] == 0xFF
        assert np.all(codes[32:96] == nan_code)
        assert scales[0] == 127 - (8 if fmt == E4M3 else 15)
        assert np.all(codes[:32] == oracle.round_with_n(np.float32(2.0 ** (8 if fmt == E4M3 else 15)), fmt, RNE, 1, 0))
        assert scales[3] == 0
