"""GPU parity: fbsr_round_format8 (generic (K, P, B; M) targets with K <= 8, the rounding modes of
Sec. II-A and both tie rules of Eq. (7)) against the CPU oracle, byte for byte."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from gpu_util import dev, first_mismatch, host

pytestmark = pytest.mark.gpu
RNE, SRFF, SRF, SRC, SRC_ODD, RNO, RNA = range(7)
FROM_BF16, FROM_FP16, FROM_FP32 = 0, 1, 2
MODES = [(RNE, 0), (RNO, 0), (RNA, 0)] + [(v, nb) for v in (SRFF, SRF, SRC, SRC_ODD) for nb in (1, 3, 4, 8, 16)]


def p3109(P):
    return (8, P, 1 << (7 - P), 0x7E, 0x7F, 0x80, 0, 0)


FORMATS = {"ocp_e4m3": (8, 4, 7, 0x7E, -1, 0x7F, 1, 1), "ocp_e5m2": (8, 3, 15, 0x7B, 0x7C, 0x7E, 1, 1),
           "ocp_e3m2": (6, 3, 3, 0x1F, -1, -1, 0, 1), "ocp_e2m3": (6, 4, 1, 0x1F, -1, -1, 0, 1), "ocp_e2m1": (4, 2, 1, 0x07, -1, -1, 0, 1),
           "binary8p1": p3109(1), "binary8p3": p3109(3), "binary8p4": p3109(4), "binary8p5": p3109(5), "binary8p7": p3109(7),
           # not published anywhere: an infinity that is not the code after M (whose code is odd), a zero bias,
           # the largest bias, the narrowest width
           "inf_apart": (8, 4, 7, 0x77, 0x7A, 0x7F, 1, 1), "bias0": (5, 2, 0, 0x0E, 0x0F, -1, 0, 0),
           "bias96": (8, 3, 96, 0x7B, 0x7C, 0x7E, 1, 1), "k2": (2, 1, 0, 1, -1, -1, 0, 1)}


def _oracle(oracle, x, src, d, variant, nbits, seed, offset, threads=16):
    cuts = np.linspace(0, x.size, threads + 1).astype(np.int64)
    with ThreadPoolExecutor(threads) as pool:
        parts = list(pool.map(lambda ab: oracle.round_format8(x[ab[0]:ab[1]], src, d, variant, nbits, seed, offset + int(ab[0])),
                              zip(cuts[:-1], cuts[1:])))
    return np.concatenate(parts)


def _inputs(rng, d, count):
    """fp32 patterns from far below the smallest subnormal to beyond M, with short mantissas (ties), the
    neighbourhoods of M, of the overflow tie and of the smallest normal / subnormal, and specials."""
    K, P, B, mx = d[:4]
    e_top = (mx >> (P - 1)) - B
    lo, hi = max(1, 127 + (1 - B) - (P - 1) - 30), min(254, 127 + e_top + 3)
    bits = rng.integers(0, 1 << 32, count, dtype=np.uint32)
    field = rng.integers(lo, hi + 1, count, dtype=np.uint32)
    b = (bits & np.uint32(0x807FFFFF)) | (field << np.uint32(23))
    b[::7] &= np.uint32(0xFFF00000)
    b[::11] &= np.uint32(0xFFFF8000)
    b[::13] &= np.uint32(0xFFFE0000)
    t_max = mx & ((1 << (P - 1)) - 1)
    M = (1.0 + t_max * 2.0 ** (1 - P)) * 2.0 ** e_top
    ulp_M = 2.0 ** (e_top - P + 1)
    pts = []
    for v in (M, M + ulp_M / 2, M + ulp_M, M + 0.75 * ulp_M, 2.0 ** (1 - B), 2.0 ** (2 - B - P), 2.0 ** (1 - B - P), 3 * 2.0 ** (-B - P)):
        u = int(np.float32(v).view(np.uint32))
        pts += [u - 2, u - 1, u, u + 1, u + 2]
    extra = np.array(pts + [0, 1, 0x007FFFFF, 0x00800000, 0x7F7FFFFF, 0x7F800000, 0x7F800001, 0x7FC00000, 0x7FFFFFFF], dtype=np.uint32)
    return np.concatenate([b, extra, extra | np.uint32(0x80000000)]).view(np.float32)


@pytest.mark.parametrize("name", sorted(FORMATS))
def test_fp32_source_every_mode(fbsr, oracle, name):
    d = FORMATS[name]
    x = _inputs(np.random.default_rng(len(name)), d, 3 * 2048 * 37 + 11)
    xd = dev(x)
    for variant, nbits in MODES:
        print("case fmt=%s variant=%d nbits=%d" % (name, variant, nbits), flush=True)
        got = host(fbsr.fbsr_round_format8(xd, FROM_FP32, d, variant, nbits, seed=21, offset=0))
        want = _oracle(oracle, x, FROM_FP32, d, variant, nbits, 21, 0)
        assert first_mismatch(got, want) is None, (name, variant, nbits, first_mismatch(got, want))


def test_random_descriptors(fbsr, oracle):
    """Sixty descriptors drawn at random (every combination of special encodings the checks allow), fp32 and
    16-bit sources, a random mode each: byte-identical to the oracle."""
    from test_oracle_format8 import random_descriptors
    rng = np.random.default_rng(77)
    codes16 = np.tile(np.arange(65536, dtype=np.uint16), 2)
    c16d = dev(codes16)
    for d in random_descriptors(rng, 60, oracle.format8_check):
        assert fbsr.format8_check(d)
        x = _inputs(rng, d, 2 * 2048 * 11 + 5)
        xd = dev(x)
        for variant, nbits in (MODES[int(rng.integers(0, len(MODES)))], MODES[int(rng.integers(3, len(MODES)))]):
            print("case d=%s variant=%d nbits=%d" % (d, variant, nbits), flush=True)
            got = host(fbsr.fbsr_round_format8(xd, FROM_FP32, d, variant, nbits, seed=3, offset=11))
            want = _oracle(oracle, x, FROM_FP32, d, variant, nbits, 3, 11)
            assert first_mismatch(got, want) is None, (d, variant, nbits, first_mismatch(got, want))
            src = int(rng.integers(0, 2))
            got = host(fbsr.fbsr_round_format8(c16d, src, d, variant, nbits, seed=3, offset=11))
            want = _oracle(oracle, codes16, src, d, variant, nbits, 3, 11)
            assert first_mismatch(got, want) is None, (d, src, variant, nbits, first_mismatch(got, want))


@pytest.mark.parametrize("src", [FROM_BF16, FROM_FP16])
@pytest.mark.parametrize("name", ["binary8p4", "binary8p3", "ocp_e2m3", "ocp_e2m1", "binary8p1", "inf_apart"])
def test_every_16_bit_source_code(fbsr, oracle, src, name):
    """All 65536 source codes, each at 32 different global indices."""
    d = FORMATS[name]
    codes = np.tile(np.arange(65536, dtype=np.uint16), 32)
    xd = dev(codes)
    for variant, nbits in [(RNE, 0), (RNO, 0), (RNA, 0), (SRFF, 3), (SRF, 3), (SRC, 3), (SRC_ODD, 3), (SRFF, 4), (SRC, 8), (SRC_ODD, 11), (SRF, 16)]:
        print("case src=%d fmt=%s variant=%d nbits=%d" % (src, name, variant, nbits), flush=True)
        got = host(fbsr.fbsr_round_format8(xd, src, d, variant, nbits, seed=5, offset=0))
        want = _oracle(oracle, codes, src, d, variant, nbits, 5, 0)
        assert first_mismatch(got, want) is None, (src, name, variant, nbits, first_mismatch(got, want))


@pytest.mark.parametrize("src", [FROM_BF16, FROM_FP16])
@pytest.mark.parametrize("name", ["binary8p4", "ocp_e4m3", "ocp_e5m2", "ocp_e2m1", "binary8p1", "inf_apart"])
def test_16_bit_sources_at_the_size_of_the_table_kernel(fbsr, oracle, src, name):
    """From 2^26 elements on, 16-bit sources with at most 8 random bits go through the kernel that tabulates the 2^15
    source magnitudes per workgroup.  All 65536 source codes (NaNs, infinities and both zeros among them) about 1024
    times each at different global indices, a tile count that leaves the last pass of 16 tiles ragged, an offset that
    leaves a head for the per-element kernel, a second input without a single NaN (every wave on the table path);
    formats with and without -0, saturating and with an infinity, one whose infinity is not the code after M (the
    table's entries above M hold the finished code); 11 random bits stay on the other kernel."""
    d = FORMATS[name]
    n = (1 << 26) + 21 * 2048 + 77
    rng = np.random.default_rng(7 + src)
    codes = np.tile(np.arange(65536, dtype=np.uint16), n // 65536 + 1)[:n]
    rng.shuffle(codes[: 1 << 20])
    nan_from = 0x7F81 if src == FROM_BF16 else 0x7C01
    clean = np.where((codes & 0x7FFF) >= nan_from, codes & 0x83FF, codes).astype(np.uint16)
    for host_x, tag in ((codes, "all codes"), (clean, "no NaN")):
        xd = dev(host_x)
        modes = [(RNE, 0), (RNA, 0), (SRFF, 3), (SRF, 1), (SRC, 3), (SRC_ODD, 4), (SRF, 8), (SRC, 2), (SRFF, 11)]
        for variant, nbits in (modes if tag == "all codes" else modes[2:6]):
            for offset in ((0, 8) if (variant, nbits) in ((SRFF, 3), (SRC, 3)) else (0,)):
                print("case src=%d fmt=%s %s variant=%d nbits=%d offset=%d" % (src, name, tag, variant, nbits, offset), flush=True)
                got = host(fbsr.fbsr_round_format8(xd, src, d, variant, nbits, seed=5, offset=offset))
                want = _oracle(oracle, host_x, src, d, variant, nbits, 5, offset)
                assert first_mismatch(got, want) is None, (src, name, tag, variant, nbits, offset, first_mismatch(got, want))


@pytest.mark.parametrize("n", [0, 1, 3, 4, 5, 31, 127, 2047, 2048, 2049, 3 * 2048 + 100])
def test_sizes_offsets_alignment(fbsr, oracle, n):
    rng = np.random.default_rng(n + 1)
    d = FORMATS["binary8p4"]
    x32 = rng.integers(0, 1 << 32, n + 8, dtype=np.uint32).view(np.float32)
    x16 = rng.integers(0, 1 << 16, n + 8, dtype=np.uint16)
    for src, host_x in ((FROM_FP32, x32), (FROM_BF16, x16), (FROM_FP16, x16)):
        xd = dev(host_x)
        for variant, nbits in ((SRFF, 3), (SRC_ODD, 6), (RNA, 0), (SRF, 1), (SRC, 16)):
            for offset in (0, 3, 128, (1 << 36) + 5):
                for shift in (0, 1, 3):
                    print("case n=%d src=%d variant=%d nbits=%d offset=%d shift=%d" % (n, src, variant, nbits, offset, shift), flush=True)
                    xs = xd[shift:shift + n] if n else xd[:0]
                    got = host(fbsr.fbsr_round_format8(xs, src, d, variant, nbits, seed=2, offset=offset))
                    want = oracle.round_format8(host_x[shift:shift + n], src, d, variant, nbits, seed=2, offset=offset)
                    assert first_mismatch(got, want) is None, first_mismatch(got, want)


def test_named_descriptors_equal_the_fixed_format_entry_points(fbsr):
    """fbsr_round / fbsr_round_from16 (hardware converts) and the generic integer path give the same bytes for the
    three formats that exist as target ids."""
    rng = np.random.default_rng(9)
    n = 1 << 22
    x = torch.from_numpy(rng.integers(0, 1 << 32, n, dtype=np.uint32).view(np.int32)).cuda().view(torch.float32)
    x16 = torch.from_numpy(rng.integers(0, 1 << 16, n, dtype=np.uint16).view(np.int16)).cuda()
    for fmt, name in ((1, "ocp_e4m3"), (2, "ocp_e5m2"), (3, "p3109_binary8p4")):
        d = fbsr.format8_named(name)
        for variant, nbits in ((RNE, 0), (SRFF, 2), (SRF, 4), (SRC, 8), (SRFF, 16), (SRC, 3)):
            print("case fmt=%s variant=%d nbits=%d" % (name, variant, nbits), flush=True)
            assert torch.equal(fbsr.fbsr_round(x, fmt, variant, nbits, seed=3, offset=77),
                               fbsr.fbsr_round_format8(x, FROM_FP32, d, variant, nbits, seed=3, offset=77))
            for src in (FROM_BF16, FROM_FP16):
                assert torch.equal(fbsr.fbsr_round_from16(x16, src, fmt, variant, nbits, seed=3, offset=77),
                                   fbsr.fbsr_round_format8(x16, src, d, variant, nbits, seed=3, offset=77))


def test_chunked_equals_whole_and_repeatable(fbsr):
    d = fbsr.format8_named("p3109_binary8p4")
    n = 5 * 2048 + 333
    x = torch.randn(n, device="cuda")
    whole = fbsr.fbsr_round_format8(x, FROM_FP32, d, SRC, 3, seed=11, offset=1000)
    assert torch.equal(whole, fbsr.fbsr_round_format8(x, FROM_FP32, d, SRC, 3, seed=11, offset=1000))
    cut = 2048 + 77
    a = fbsr.fbsr_round_format8(x[:cut], FROM_FP32, d, SRC, 3, seed=11, offset=1000)
    b = fbsr.fbsr_round_format8(x[cut:], FROM_FP32, d, SRC, 3, seed=11, offset=1000 + cut)
    assert torch.equal(whole, torch.cat([a, b]))


def test_sec4_training_cast_bias_on_the_gpu(fbsr, oracle):
    """Sec. IV's cast, bf16 updates -> binary8p4 with 3 random bits (D = 4 excess bits), at scale: every
    bf16 value of [1, 2), 2^15 draws each.  Mean error in target ulps: SRFF (2^-4 - 2^-3)/2 = -0.03125,
    SRF +2^-5 = +0.03125, SRC (either tie rule) 0, within the noise of the draws (0.3 / sqrt(4.2e6))."""
    d = FORMATS["binary8p4"]
    draws = 1 << 15
    codes = np.repeat(np.arange(0x3F80, 0x4000, dtype=np.uint16), draws)
    xd = dev(codes)
    xv = (codes.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    table = np.array([oracle.decode_format8(c, d) for c in range(256)])
    for variant, want in ((SRFF, -0.03125), (SRF, 0.03125), (SRC, 0.0), (SRC_ODD, 0.0)):
        got = host(fbsr.fbsr_round_format8(xd, FROM_BF16, d, variant, 3, seed=31, offset=0))
        bias = np.mean((table[got] - xv) / 0.125)
        print("variant=%d bias=%+.6f ulp (closed form %+.6f)" % (variant, bias, want), flush=True)
        assert abs(bias - want) < 1e-3
    sample = slice(0, codes.size, 257)
    want_codes = oracle.round_format8(codes, FROM_BF16, d, SRFF, 3, 31, 0)
    got = host(fbsr.fbsr_round_format8(xd, FROM_BF16, d, SRFF, 3, seed=31, offset=0))
    assert np.array_equal(got[sample], want_codes[sample])


def test_rejects_bad_arguments(fbsr):
    x = torch.zeros(16, device="cuda")
    good = FORMATS["binary8p4"]
    for d, variant, nbits in (((8, 4, 8, 0x7E, 0x7E, 0x80, 0, 0), SRFF, 3), (good, 7, 3), (good, SRC_ODD, 25), (good, SRF, 0)):
        with pytest.raises(fbsr.FbsrError):
            fbsr.fbsr_round_format8(x, FROM_FP32, d, variant, nbits, seed=0)


@pytest.mark.parametrize("name,variant,nbits", [("binary8p4", SRC_ODD, 3), ("ocp_e2m1", SRF, 2), ("binary8p3", RNA, 0),
                                                 ("binary8p4", SRC_ODD, 23), ("binary8p7", SRF, 24), ("ocp_e2m1", SRC, 24)])
def test_every_fp32_pattern_generic(fbsr, oracle, name, variant, nbits):
    """All 2^32 input patterns through the generic tile kernel, in 16 slabs of 2^28: byte-identical to the oracle.  The
    cases with more than 16 bits are the corners of that rounding in the 24-bit code space: the inner rounding's tie at
    the code space's last place, the half step below it, no bit dropped at all."""
    d = FORMATS[name]
    slab = 1 << 28
    for s_no in range(16):
        base = s_no * slab
        x = np.arange(base, base + slab, dtype=np.uint32).view(np.float32)
        lo = base - (1 << 32) if base >= (1 << 31) else base
        xd = torch.arange(lo, lo + slab, dtype=torch.int64, device="cuda").to(torch.int32).view(torch.float32)
        got = host(fbsr.fbsr_round_format8(xd, FROM_FP32, d, variant, nbits, seed=77, offset=base))
        del xd
        want = _oracle(oracle, x, FROM_FP32, d, variant, nbits, 77, base)
        print("case fmt=%s variant=%d nbits=%d slab=%d" % (name, variant, nbits, s_no), flush=True)
        assert first_mismatch(got, want) is None, (s_no, first_mismatch(got, want))
